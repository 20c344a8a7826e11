"""Pins for the oracle's compositions: one block (select_block), the indicator average (lsh_scores) and
the layer loop's look-back wiring (compress_layer).  Alg. 1 steps 3-8; Sec. 3.1; Sec. 3.2.

The one-block example is worked by hand: d = 2, one look-back key, six block keys, two query heads of
one KV head with a window of two queries, two one-bit tables.  Queries are c * (integer vector) with
c = sqrt(2) ln 2, so a logit q.k / sqrt(2) is (integer dot product) * ln 2 and every softmax weight is
a power of two; all probabilities below are exact fractions.
"""
from fractions import Fraction as F

import numpy as np
import pytest

from oracle import laserkv_oracle as O

C = np.sqrt(2.0) * np.log(2.0)
K_BLK = [(-1, 1), (-1, 2), (-2, 0), (2, 2), (-1, -2), (-2, 1)]     # positions 0..5
K_CTX = [(-1, -1)]                                                  # look-back key: always visible
Q_WIN = [[(-1, 2), (0, 1)],                                         # query head 0: window queries at positions 4, 5
         [(2, -1), (2, -2)]]                                        # query head 1
PLANES = [(1.0, 0.25), (1.0, -1.5)]                                 # table 0 / table 1, one sign bit each

# Weights 2^(q.k) per row over [ctx, k0..k5]; the query at position 4 does not see k5.
#   (-1, 2): ctx 2^-1, k0 2^3, k1 2^5, k2 2^2, k3 2^2, k4 2^-3            sum 389/8
#   ( 0, 1): ctx 2^-1, k0 2^1, k1 2^2, k2 2^0, k3 2^2, k4 2^-2, k5 2^1    sum 55/4
#   ( 2,-1): ctx 2^-1, k0 2^-3, k1 2^-4, k2 2^-4, k3 2^2, k4 2^0          sum 92/16
#   ( 2,-2): ctx 2^0, k0 2^-4, k1 2^-6, k2 2^-4, k3 2^0, k4 2^2, k5 2^-6  sum 394/64
ROW_PROBS = [
    [F(64, 389), F(256, 389), F(32, 389), F(32, 389), F(1, 389), F(0)],
    [F(8, 55), F(16, 55), F(4, 55), F(16, 55), F(1, 55), F(8, 55)],
    [F(2, 92), F(1, 92), F(1, 92), F(64, 92), F(16, 92), F(0)],
    [F(4, 394), F(1, 394), F(4, 394), F(64, 394), F(256, 394), F(1, 394)],
]
S_EXACT = [sum(r[i] for r in ROW_PROBS) / 4 for i in range(6)]      # mean over the G*W = 4 rows
# Sign bits (projection >= 0).  Table 0, x + y/4: keys 0 0 0 1 0 0; queries (-1,2) 0, (0,1) 1, (2,-1) 1, (2,-2) 1.
#                               Table 1, x - 3y/2: keys 0 0 0 0 1 0; queries 0, 0, 1, 1.
SIG_K = [[0, 0], [0, 0], [0, 0], [1, 0], [0, 1], [0, 0]]
SIG_Q = [[[0, 0], [1, 0]], [[1, 1], [1, 1]]]
# Table 0: one query has code 0, three have code 1 -> keys with code 0 collide once, k3 three times.
# Table 1: two and two -> every key collides twice.
CNT = [3, 3, 3, 5, 3, 3]
# Partition: 1 anchor (k0), 1 local (k5), candidates k1..k4, k_exact = 2, k_lsh = 1.
# Stage 1: scores k1 .2406, k2 .0440, k3 .3078, k4 .2111 -> {k3, k1}.
# Stage 2: residual {k2, k4}, counts tie at 3 -> lower index k2 (although k4 scores higher).
KEEP = [0, 1, 2, 3, 5]


def _block():
    q = np.asarray(Q_WIN, dtype=np.float64) * C
    return q, np.asarray([K_BLK], dtype=np.float64), np.asarray([K_CTX], dtype=np.float64), np.asarray(PLANES)


def test_select_block_hand_worked_example():
    q, k, kc, planes = _block()
    st = O.select_block(q, k, kc, planes, 2, 1, 1, 1, 2, 1, block_pos0=0)
    np.testing.assert_allclose(st["s_exact"][0], [float(x) for x in S_EXACT], rtol=1e-13)
    assert float(sum(S_EXACT)) < 1.0                                # the look-back key took its share
    assert st["sig_k"][0].tolist() == SIG_K
    assert st["sig_q"].tolist() == SIG_Q
    assert not st["unsure_k"].any() and not st["unsure_q"].any()
    assert st["cnt"][0].tolist() == CNT
    assert st["k_exact_set"][0].tolist() == [1, 3]
    assert st["k_lsh_set"][0].tolist() == [2]
    assert st["keep"][0].tolist() == KEEP
    # the same block at another absolute position (default window = its last W tokens): nothing changes
    st2 = O.select_block(q, k, kc, planes, 2, 1, 1, 1, 2, 1, block_pos0=1000)
    assert st2["keep"][0].tolist() == KEEP
    # each ingredient matters in this example: no look-back key, no mask, or no stage 2 give other sets
    assert O.select_block(q, k, None, planes, 2, 1, 1, 1, 2, 1)["keep"][0].tolist() != KEEP
    assert O.select_block(q, k, kc, planes, 2, 1, 1, 1, 2, 1, causal=False)["keep"][0].tolist() != KEEP
    assert O.select_block(q, k, kc, planes, 2, 1, 1, 1, 3, 0)["keep"][0].tolist() == [0, 1, 3, 4, 5]


def test_lsh_scores_literal():
    # Alg. 1 step 6: average of the indicators over G * W * R = 2 * 2 * 2 = 8 (query, table) pairs
    assert O.lsh_scores(CNT, 2, 2, 2).tolist() == [0.375, 0.375, 0.375, 0.625, 0.375, 0.375]
    assert O.lsh_scores([0, 8], 2, 2, 2).tolist() == [0.0, 1.0]


def test_select_block_keeps_each_kv_head_with_its_own_query_heads():
    """Two KV heads, G = 2: head h must be scored and counted with query heads 2h and 2h + 1 only."""
    q, k, kc, planes = _block()
    rng = np.random.default_rng(3)
    k_other = rng.integers(-2, 3, size=(1, 6, 2)).astype(np.float64) + 0.125
    q_other = (rng.integers(-2, 3, size=(2, 2, 2)).astype(np.float64) + 0.125) * C
    kc_other = np.asarray([[(1.0, 2.0)]])
    both = O.select_block(np.concatenate([q_other, q]), np.concatenate([k_other, k]), np.concatenate([kc_other, kc]),
                          planes, 2, 1, 1, 1, 2, 1)
    alone = O.select_block(q_other, k_other, kc_other, planes, 2, 1, 1, 1, 2, 1)
    np.testing.assert_allclose(both["s_exact"][1], [float(x) for x in S_EXACT], rtol=1e-13)
    assert both["cnt"][1].tolist() == CNT and both["keep"][1].tolist() == KEEP
    np.testing.assert_array_equal(both["s_exact"][0], alone["s_exact"][0])
    assert both["cnt"][0].tolist() == alone["cnt"][0].tolist()
    assert both["keep"][0].tolist() == alone["keep"][0].tolist()


def test_compress_layer_look_back_is_the_previous_blocks_local_window():
    """Sec. 3.2: block t is scored with the tail of block t-1 as context-only keys.  Re-derive every block
    from the RAW keys (the previous block's last n_local rows) and compare all stages; block lengths are
    chosen so that consecutive blocks have different n_local (B_t = min(B, S_t))."""
    rng = np.random.default_rng(11)
    h_q, h_kv, d, w, L, Kb = 4, 2, 8, 4, 3, 4
    lens = [40, 16, 28, 40]
    B, n, alpha = 24, 4, 0.75
    n_local = [O.partition(B, n, alpha, s)[1] for s in lens]
    assert n_local == [6, 4, 6, 6]
    total = sum(lens)
    k = rng.standard_normal((h_kv, total, d))
    v = rng.standard_normal((h_kv, total, d))
    planes = rng.standard_normal((L * Kb, d))
    qs = [rng.standard_normal((h_q, w, d)) * 2.0 for _ in lens]
    starts = np.concatenate([[0], np.cumsum(lens)[:-1]])
    blocks = [(qs[t], k[:, lo:lo + s], v[:, lo:lo + s], int(lo)) for t, (lo, s) in enumerate(zip(starts, lens))]
    ck, cv, cp, clen, stages = O.compress_layer(blocks, planes, L, Kb, B, n, alpha, cap=sum(min(B, s) for s in lens))
    assert clen == sum(min(B, s) for s in lens)
    for t, (lo, s) in enumerate(zip(starts, lens)):
        parts = O.partition(B, n, alpha, s)
        k_ctx = k[:, lo - n_local[t - 1]:lo] if t else None       # tail of block t-1, from the raw keys
        st = O.select_block(qs[t], k[:, lo:lo + s], k_ctx, planes, L, Kb, *parts, block_pos0=int(lo))
        np.testing.assert_array_equal(st["s_exact"], stages[t]["s_exact"])
        np.testing.assert_array_equal(st["cnt"], stages[t]["cnt"])
        np.testing.assert_array_equal(st["keep"], stages[t]["keep"])
        if t:
            # the look-back keys matter: another tail length, or none, changes the scores
            for wrong in (k[:, lo - n_local[t]:lo] if n_local[t] != n_local[t - 1] else None, None):
                alt = O.exact_scores(qs[t], k[:, lo:lo + s], wrong, block_pos0=int(lo))
                assert np.abs(alt - stages[t]["s_exact"]).max() > 1e-6
    # the cache holds the kept rows of every block in order, positions absolute
    off = 0
    for t, (lo, s) in enumerate(zip(starts, lens)):
        b_t = min(B, s)
        for h in range(h_kv):
            np.testing.assert_array_equal(cp[h, off:off + b_t], lo + stages[t]["keep"][h])
            np.testing.assert_array_equal(ck[h, off:off + b_t], k[h, lo + stages[t]["keep"][h]])
            np.testing.assert_array_equal(cv[h, off:off + b_t], v[h, lo + stages[t]["keep"][h]])
        off += b_t


def _layer_inputs(seed, lens, h_q=4, h_kv=2, d=8, w=4, L=3, Kb=4):
    rng = np.random.default_rng(seed)
    total = sum(lens)
    k = rng.standard_normal((h_kv, total, d))
    v = rng.standard_normal((h_kv, total, d))
    planes = rng.standard_normal((L * Kb, d))
    qs = [rng.standard_normal((h_q, w, d)) * 2.0 for _ in lens]
    starts = [int(x) for x in np.concatenate([[0], np.cumsum(lens)[:-1]])]
    blocks = [(qs[t], k[:, lo:lo + s], v[:, lo:lo + s], lo) for t, (lo, s) in enumerate(zip(starts, lens))]
    return k, v, planes, qs, starts, blocks, L, Kb, w


def test_deferred_tail_of_zero_is_the_plain_layer_loop():
    lens = [40, 16, 28, 40]
    k, v, planes, qs, starts, blocks, L, Kb, w = _layer_inputs(5, lens)
    B, n, alpha = 24, 4, 0.75
    cap = sum(min(B, s) for s in lens)
    a = O.compress_layer(blocks, planes, L, Kb, B, n, alpha, cap=cap)
    b = O.compress_layer_deferred(blocks, planes, L, Kb, B, n, alpha, cap=cap, tail=0)
    assert a[3] == b[3]
    for x, y in zip(a[:3], b[:3]):
        np.testing.assert_array_equal(x, y)
    for sa, sb in zip(a[4], b[4]):
        np.testing.assert_array_equal(sa["s_exact"], sb["s_exact"])
        np.testing.assert_array_equal(sa["keep"], sb["keep"])


def test_deferred_tail_segments_follow_sec_3_2():
    """Every segment re-derived from the raw tensors: it starts `tail` tokens before its block, ends `tail`
    tokens before the block's end (the last block ends with its block), is scored by the block's own last W
    tokens at their real positions, and sees the previous segment's local window as context-only keys."""
    lens, tail = [40, 24, 40, 32], 6
    k, v, planes, qs, starts, blocks, L, Kb, w = _layer_inputs(6, lens)
    B, n, alpha = 24, 4, 0.75
    total = sum(lens)
    seg_lo = [0] + [starts[t] - tail for t in range(1, len(lens))]
    seg_hi = [starts[t] + lens[t] - tail for t in range(len(lens) - 1)] + [total]
    cap = sum(min(B, hi - lo) for lo, hi in zip(seg_lo, seg_hi))
    ck, cv, cp, clen, stages = O.compress_layer_deferred(blocks, planes, L, Kb, B, n, alpha, cap=cap, tail=tail)
    assert clen == cap                                                   # kept count = budget of every segment
    assert seg_hi[:-1] == seg_lo[1:]                                     # the segments tile the context: each token is judged once
    n_local_prev = 0
    off = 0
    for t, (lo, hi) in enumerate(zip(seg_lo, seg_hi)):
        parts = O.partition(B, n, alpha, hi - lo)
        assert stages[t]["seg_pos0"] == lo and stages[t]["seg_len"] == hi - lo
        k_ctx = k[:, lo - n_local_prev:lo] if t else None               # raw keys just before the segment
        st = O.select_block(qs[t], k[:, lo:hi], k_ctx, planes, L, Kb, *parts, block_pos0=lo,
                            q_pos0=starts[t] + lens[t] - w)
        np.testing.assert_array_equal(st["s_exact"], stages[t]["s_exact"])
        np.testing.assert_array_equal(st["cnt"], stages[t]["cnt"])
        np.testing.assert_array_equal(st["keep"], stages[t]["keep"])
        b_t = sum(parts)
        for h in range(k.shape[0]):
            np.testing.assert_array_equal(cp[h, off:off + b_t], lo + st["keep"][h])
            np.testing.assert_array_equal(ck[h, off:off + b_t], k[h, lo + st["keep"][h]])
            np.testing.assert_array_equal(cv[h, off:off + b_t], v[h, lo + st["keep"][h]])
        if t < len(lens) - 1:
            # the block's own tail is judged later: none of it is in the cache yet, and the window's last
            # `tail` queries lie beyond the segment, so the mask hides fewer keys than in the plain loop
            assert cp[:, :off + b_t].max() < hi
            plain = O.exact_scores(qs[t], k[:, lo:hi], k_ctx, block_pos0=lo)   # window = the SEGMENT's last W tokens
            assert np.abs(plain - st["s_exact"]).max() > 1e-6
        off += b_t
        n_local_prev = parts[1]
    assert np.all(np.diff(cp[:, :clen], axis=1) > 0)                     # append-only order
    with pytest.raises(ValueError):
        O.compress_layer_deferred(blocks, planes, L, Kb, B, n, alpha, cap=cap, tail=25)
