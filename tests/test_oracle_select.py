"""Pins for the oracle's Exact-LSH selection (Alg. 1 steps 4-8; Sec. 3.1 partition) and the append."""
import itertools

import numpy as np
import pytest
import torch

from oracle import laserkv_oracle as O


def _greedy_pick(cands, score, k):
    """Independent definition of TopK with lower-index tie-break: k rounds of 'take the best remaining'."""
    left = list(cands)
    out = []
    for _ in range(k):
        best = left[0]
        for i in left[1:]:
            if score[i] > score[best] or (score[i] == score[best] and i < best):
                best = i
        out.append(best)
        left.remove(best)
    return out


@pytest.mark.parametrize("seed", range(12))
def test_selection_matches_greedy_definition_with_heavy_ties(seed):
    rng = np.random.default_rng(seed)
    s = int(rng.integers(12, 40))
    a = int(rng.integers(0, 4))
    loc = int(rng.integers(0, 4))
    n_c = s - a - loc
    ke = int(rng.integers(0, n_c // 2 + 1))
    kl = int(rng.integers(0, n_c - ke + 1))
    s_exact = rng.integers(0, 4, s) / 8.0                 # few distinct values: ties everywhere
    cnt = rng.integers(0, 3, s)
    keep, k_ex, k_l = O.select(s_exact, cnt, a, loc, ke, kl)
    cands = list(range(a, s - loc))
    ref_ex = _greedy_pick(cands, s_exact, ke)
    resid = [i for i in cands if i not in ref_ex]
    ref_l = _greedy_pick(resid, cnt, kl)
    assert sorted(ref_ex) == k_ex.tolist() and sorted(ref_l) == k_l.tolist()
    assert keep.tolist() == sorted(set(range(a)) | set(range(s - loc, s)) | set(ref_ex) | set(ref_l))


def test_selection_invariants_and_library_topk_without_ties():
    rng = np.random.default_rng(100)
    s, a, loc, ke, kl = 300, 20, 25, 60, 30
    s_exact = rng.random(s)
    cnt = rng.permutation(s)                                # all distinct: TopK is unique
    keep, k_ex, k_l = O.select(s_exact, cnt, a, loc, ke, kl)
    assert len(keep) == a + loc + ke + kl                   # kept count == budget
    assert np.all(np.diff(keep) > 0)                        # ascending => no duplicates
    assert set(range(a)) <= set(keep) and set(range(s - loc, s)) <= set(keep)
    assert not (set(k_ex) & set(k_l))
    cand = np.arange(a, s - loc)
    top = torch.topk(torch.from_numpy(s_exact[cand]), ke).indices.numpy() + a
    assert sorted(top.tolist()) == k_ex.tolist()
    resid = np.array([i for i in cand if i not in set(k_ex.tolist())])
    top2 = resid[torch.topk(torch.from_numpy(cnt[resid]), kl).indices.numpy()]
    assert sorted(top2.tolist()) == k_l.tolist()
    # threshold property: nothing left out beats anything taken, stage by stage
    out1 = np.setdiff1d(cand, k_ex)
    assert s_exact[out1].max() < s_exact[k_ex].min()
    out2 = np.setdiff1d(resid, k_l)
    assert cnt[out2].max() < cnt[k_l].min()


def test_alpha_end_points_degenerate_to_single_metric_topk():
    # alpha = 1: pure attention TopK ("Exact" row of Table 1); alpha = 0: pure collision TopK ("MagicPIG" row).
    rng = np.random.default_rng(7)
    s, B, n = 200, 80, 4
    s_exact = rng.random(s)
    cnt = rng.integers(0, 50, s)
    a, loc, ke, kl = O.partition(B, n, 1.0, s)
    keep, k_ex, k_l = O.select(s_exact, cnt, a, loc, ke, kl)
    cand = np.arange(a, s - loc)
    order = cand[np.lexsort((cand, -s_exact[cand]))]
    assert len(k_l) == 0 and k_ex.tolist() == sorted(order[:ke].tolist())
    a, loc, ke, kl = O.partition(B, n, 0.0, s)
    keep, k_ex, k_l = O.select(s_exact, cnt, a, loc, ke, kl)
    order = cand[np.lexsort((cand, -cnt[cand]))]
    assert len(k_ex) == 0 and k_l.tolist() == sorted(order[:kl].tolist())


def test_stage_two_ranks_only_the_residual():
    # token 3 wins both metrics: it must be taken by stage 1 and not consume a stage-2 slot.
    s_exact = np.array([0, 0, 0.1, 0.9, 0.2, 0.3, 0, 0], dtype=float)
    cnt = np.array([0, 0, 5, 9, 1, 7, 0, 0])
    keep, k_ex, k_l = O.select(s_exact, cnt, 1, 1, 1, 2)
    assert k_ex.tolist() == [3] and k_l.tolist() == [2, 5] and keep.tolist() == [0, 2, 3, 5, 7]


def test_select_rejects_oversized_budgets():
    with pytest.raises(ValueError):
        O.select(np.zeros(10), np.zeros(10, int), 6, 6, 0, 0)
    with pytest.raises(ValueError):
        O.select(np.zeros(10), np.zeros(10, int), 2, 2, 4, 3)


def test_append_is_bit_exact_append_only_and_ordered():
    rng = np.random.default_rng(8)
    hkv, cap, d = 2, 64, 4
    ck = np.zeros((hkv, cap, d)); cv = np.zeros((hkv, cap, d)); cp = np.full((hkv, cap), -1, dtype=np.int64)
    length = 0
    snapshots = []
    for t in range(3):
        s = 20
        kb = rng.standard_normal((hkv, s, d)); vb = rng.standard_normal((hkv, s, d))
        keep = np.stack([np.sort(rng.choice(s, 7, replace=False)) for _ in range(hkv)])
        new_len = O.append(ck, cv, cp, length, kb, vb, keep, 1000 + t * s)
        assert new_len == length + 7
        for h in range(hkv):
            assert np.array_equal(ck[h, length:new_len], kb[h, keep[h]])
            assert np.array_equal(cv[h, length:new_len], vb[h, keep[h]])
            assert np.array_equal(cp[h, length:new_len], 1000 + t * s + keep[h])
        for (l0, k0, v0, p0) in snapshots:                  # earlier rows untouched
            assert np.array_equal(ck[:, :l0], k0) and np.array_equal(cv[:, :l0], v0) and np.array_equal(cp[:, :l0], p0)
        length = new_len
        snapshots.append((length, ck[:, :length].copy(), cv[:, :length].copy(), cp[:, :length].copy()))
    assert np.all(np.diff(cp[:, :length], axis=1) > 0) and np.all(cp[:, length:] == -1)
    with pytest.raises(ValueError):
        O.append(ck, cv, cp, 60, kb, vb, keep, 0)
