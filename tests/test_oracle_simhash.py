"""Pins for the oracle's SimHash signatures and collision counts (Sec. 3.3 "Recall"; Alg. 1 step 6)."""
import math

import numpy as np
import pytest

from oracle import laserkv_oracle as O


def _pair_at_cos(d, c, rng):
    a = rng.standard_normal(d)
    b = rng.standard_normal(d)
    a /= np.linalg.norm(a)
    b -= (b @ a) * a
    b /= np.linalg.norm(b)
    return a * 3.7, (c * a + math.sqrt(1 - c * c) * b) * 0.2     # norms differ on purpose


def test_bit_order_and_table_layout_by_inspection():
    # planes are signed unit vectors, so every bit can be read off x by eye.
    x = np.array([1.0, -2.0, 3.0, -4.0])
    e = np.eye(4)
    planes = np.stack([e[1], e[0], e[2], e[3], -e[3], -e[0]])     # L = 3 tables x K = 2 bits
    sig, unsure = O.simhash(x, planes, 3, 2)
    # table 0: bit0 = [x1>=0]=0, bit1 = [x0>=0]=1 -> 2 ; table 1: bit0=[x2>=0]=1, bit1=[x3>=0]=0 -> 1
    # table 2: bit0 = [-x3>=0]=1, bit1=[-x0>=0]=0 -> 1
    assert sig.tolist() == [2, 1, 1] and not unsure.any()


def test_zero_projection_sets_the_bit_and_is_flagged():
    sig, unsure = O.simhash(np.zeros(8), np.random.default_rng(0).standard_normal((12, 8)), 3, 4)
    assert sig.tolist() == [15, 15, 15] and unsure.all()
    x = np.array([1.0, 0.0])
    planes = np.array([[5e-4, 1.0], [1.0, 0.0]])                 # first projection 5e-4: below the threshold
    sig, unsure = O.simhash(x, planes, 2, 1)
    assert sig.tolist() == [1, 1] and unsure.tolist() == [True, False]


def test_positive_scale_invariance_and_negation():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((50, 32))
    planes = rng.standard_normal((6 * 10, 32))
    sig, _ = O.simhash(x, planes, 6, 10)
    for c in (1e-3, 0.5, 7.0, 1e4):
        sig_c, _ = O.simhash(c * x, planes, 6, 10)
        assert np.array_equal(sig, sig_c)
    neg, _ = O.simhash(-x, planes, 6, 10)
    assert np.array_equal(neg, (2 ** 10 - 1) - sig)               # bitwise complement (no projection is 0)


@pytest.mark.parametrize("c", [0.9, 0.99, 0.0, -0.5])
def test_bit_agreement_rate_is_one_minus_theta_over_pi(c):
    # Random-hyperplane closed form: P[bit equal] = 1 - theta / pi.
    rng = np.random.default_rng(2)
    d, n_tables, n_bits = 64, 25000, 8
    a, b = _pair_at_cos(d, c, rng)
    planes = rng.standard_normal((n_tables * n_bits, d))
    sa, _ = O.simhash(a, planes, n_tables, n_bits)
    sb, _ = O.simhash(b, planes, n_tables, n_bits)
    x = sa ^ sb
    n_diff = sum(int(((x >> bit) & 1).sum()) for bit in range(n_bits))
    n = n_tables * n_bits
    p = 1 - math.acos(c) / math.pi
    assert abs((n - n_diff) / n - p) < 4 * math.sqrt(p * (1 - p) / n)
    # per-table collision rate: (1 - theta/pi)^K
    pk = p ** n_bits
    rate = float((sa == sb).mean())
    assert abs(rate - pk) < 4 * math.sqrt(pk * (1 - pk) / n_tables) + 1e-12


def test_closed_form_values_quoted_for_the_workloads():
    p = lambda c: 1 - math.acos(c) / math.pi
    assert abs(p(0.9) - 0.85643) < 1e-5 and abs(p(0.99) - 0.95495) < 1e-5
    assert abs(p(0.9) ** 12 - 0.1557) < 1e-4 and abs(p(0.9) ** 16 - 0.0838) < 1e-4


def test_counts_match_triple_loop():
    rng = np.random.default_rng(3)
    hq, hkv, w, s, n_tables = 6, 3, 5, 40, 4
    g = hq // hkv
    sig_q = rng.integers(0, 4, (hq, w, n_tables))      # 2-bit codes: many collisions
    sig_k = rng.integers(0, 4, (hkv, s, n_tables))
    got = O.collision_counts(sig_q, sig_k, g)
    for h in range(hkv):
        for i in range(s):
            c = 0
            for gg in range(g):
                for j in range(w):
                    for r in range(n_tables):
                        c += int(sig_q[h * g + gg, j, r] == sig_k[h, i, r])
            assert got[h, i] == c
    assert got.min() >= 0 and got.max() <= g * w * n_tables


def test_counts_group_mapping_and_duplicates():
    # Only query head 3 (= KV head 1, group member 1 when G = 2) can collide.
    sig_q = np.full((4, 2, 3), 99)
    sig_q[3, :, :] = 7
    sig_k = np.zeros((2, 5, 3), dtype=np.int64)
    sig_k[1, 2, :] = 7
    sig_k[0, 2, :] = 7
    cnt = O.collision_counts(sig_q, sig_k, 2)
    assert cnt[1, 2] == 2 * 3 and cnt.sum() == 6
    # identical keys get identical counts; a key equal to a query collides in every table
    rng = np.random.default_rng(4)
    planes = rng.standard_normal((8 * 6, 16))
    q = rng.standard_normal((2, 4, 16))
    k = rng.standard_normal((1, 10, 16))
    k[0, 7] = k[0, 2]
    k[0, 5] = 2.5 * q[1, 3]
    sq, _ = O.simhash(q, planes, 8, 6)
    sk, _ = O.simhash(k, planes, 8, 6)
    cnt = O.collision_counts(sq, sk, 2)
    assert cnt[0, 7] == cnt[0, 2] and cnt[0, 5] >= 8


def test_collision_rate_of_counts_matches_closed_form():
    # One query, keys at cos 0.9 to it: per key, cnt / L -> (1 - theta/pi)^K over independent tables;
    # unrelated random keys -> 2^-K.
    rng = np.random.default_rng(5)
    d, n_tables, n_bits, n_keys = 32, 6000, 6, 20
    q = rng.standard_normal(d)
    qh = q / np.linalg.norm(q)
    keys = []
    for _ in range(n_keys):
        v = rng.standard_normal(d)
        v -= (v @ qh) * qh
        keys.append((0.9 * qh + math.sqrt(0.19) * v / np.linalg.norm(v)) * rng.uniform(0.1, 9.0))
    keys = np.stack(keys)
    planes = rng.standard_normal((n_tables * n_bits, d))
    sq, _ = O.simhash(q[None, None, :], planes, n_tables, n_bits)
    sk, _ = O.simhash(keys[None], planes, n_tables, n_bits)
    cnt = O.collision_counts(sq, sk, 1)[0]
    pk = (1 - math.acos(0.9) / math.pi) ** n_bits
    assert np.all(np.abs(cnt / n_tables - pk) < 4.5 * math.sqrt(pk * (1 - pk) / n_tables))
    rnd = rng.standard_normal((1, n_keys, d))
    sr, _ = O.simhash(rnd, planes, n_tables, n_bits)
    cr = O.collision_counts(sq, sr, 1)[0]
    # a random key sits at its own angle to q: compare with that key's closed form
    cosr = (rnd[0] @ qh) / np.linalg.norm(rnd[0], axis=1)
    pr = (1 - np.arccos(cosr) / math.pi) ** n_bits
    assert np.all(np.abs(cr / n_tables - pr) < 4.5 * np.sqrt(pr * (1 - pr) / n_tables))
    s_lsh = O.lsh_scores(cnt, 1, 1, n_tables)
    assert 0 <= s_lsh.min() and s_lsh.max() <= 1 and abs(s_lsh.mean() - pk) < 0.01


def test_one_bit_tables_give_the_hamming_score():
    """With K = 1 every table is one sign bit, and the collision count of a key is
    G*W*L minus the summed Hamming distance between its bit string and the window queries'
    (the bit-wise reading of the hash score)."""
    rng = np.random.default_rng(11)
    h_q, h_kv, w, s_t, d, L = 4, 2, 5, 30, 16, 24
    planes = rng.standard_normal((L, d))
    q = rng.standard_normal((h_q, w, d))
    k = rng.standard_normal((h_kv, s_t, d))
    sig_q, _ = O.simhash(q, planes, L, 1)
    sig_k, _ = O.simhash(k, planes, L, 1)
    cnt = O.collision_counts(sig_q, sig_k, h_q // h_kv)
    g = h_q // h_kv
    for h in range(h_kv):
        bits_k = (k[h] @ planes.T >= 0)
        for i in range(s_t):
            ham = 0
            for gi in range(g):
                bits_q = (q[h * g + gi] @ planes.T >= 0)
                ham += int((bits_q != bits_k[i][None, :]).sum())
            assert cnt[h, i] == g * w * L - ham
