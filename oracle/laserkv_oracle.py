"""CPU oracle for LASER-KV's block-wise prefill KV selection.

TEST INFRASTRUCTURE ONLY.  This module is the slow, plain definition that the
HIP path is checked against.  Only the test-suite, the smoke check and the
benchmark's CPU-baseline leg may import it; the product never does, and this
module imports nothing from the product.

Everything is NumPy float64 (integers for counts and indices).  Inputs are the
storage-precision values (bf16 / fp32) promoted to float64 by the caller.

Notation follows the paper where it does not clash:
  S_t      tokens in the current block B_t             (Sec. 3.2)
  B        per-block, per-head budget                  (Sec. 3.1, App. B eq.)
  n        protection divisor                          (Sec. 3.1)
  alpha    exact share of the recall budget B_long     (Alg. 1 input)
  R        number of hash functions h_r; here each h_r is one table's
           K_bits-bit random-hyperplane (SimHash) code (Sec. 3.3 "Recall")
  W        observation-window length = query length L_q (Sec. 3.3 "Precision")
  G        query heads per KV head (grouped-query attention)
  T        look-back keys taken from the tail of block t-1 (Sec. 3.2)

Readings taken where the paper is silent (each is listed in the design notes):
  * Attn(Q, C) is the softmax over [look-back keys | block keys] with a causal
    mask on block keys, and the probabilities are averaged (sum / (G*W)) over
    the window queries and the GQA group of one KV head.
  * h_r(Q) = h_r(k) is evaluated for every window query separately and the
    indicators are summed over (group member, window query, table).
  * sign(0) counts as a set bit (projection >= 0).
  * TopK breaks ties towards the lower token index.
  * Every block keeps its first floor(B/n) and last floor(B/n) tokens.

  * Global-consensus variant (consensus_block): Alg. 1 step 3 taken literally,
    S_exact summed over every layer and head handed in, and likewise the
    collision counts of step 6, then ONE selection shared by all of them.

  * Attention over the compacted cache (attend_cache): plain softmax attention
    of later queries over the kept rows, every kept row visible.

Pins: see tests/test_oracle_*.py.  The composition of the steps into one
layer-level run (compress_layer) has no printed worked example in the paper:
whole-path parity unpinned beyond the per-step pins and the invariants.
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np

UNSURE_EPS = 1e-3  # |projection| below this: the sign bit is not compared


# --------------------------------------------------------------------------
# a0  budget and partition (Sec. 3.1; App. B equation)
# --------------------------------------------------------------------------
def budget(s_block: int, l_ctx: int, r_num: int = 1, r_den: int = 4) -> int:
    """Per-block budget B = floor(2 r S L / (S + L)), r = r_num / r_den.

    App. B equation; evaluated in exact rational arithmetic.
    """
    r = Fraction(int(r_num), int(r_den))
    val = 2 * r * int(s_block) * int(l_ctx) / (int(s_block) + int(l_ctx))
    return int(val.numerator // val.denominator)


def partition(B: int, n: int, alpha: float, s_t: int):
    """Split a block's budget (Sec. 3.1, Alg. 1 steps 4 and 7).

    Returns (n_anchor, n_local, k_exact, k_lsh) with
      B_t     = min(B, s_t)
      n_anchor = n_local = floor(B_t / n)          "B/n" each
      B_long  = B_t - 2 floor(B_t / n)             "B - 2B/n"
      k_exact = floor(alpha * B_long)              "alpha * B_long"
      k_lsh   = B_long - k_exact                   "(1 - alpha) * B_long"
    so that the four always sum to B_t.
    """
    if n < 2:
        raise ValueError("protection divisor n must be >= 2")
    if not (0.0 <= alpha <= 1.0):
        raise ValueError("alpha must lie in [0, 1]")
    b_t = min(int(B), int(s_t))
    a = b_t // int(n)
    b_long = b_t - 2 * a
    k_exact = int(np.floor(np.float64(alpha) * np.float64(b_long)))
    k_lsh = b_long - k_exact
    return a, a, k_exact, k_lsh


# --------------------------------------------------------------------------
# a1  exact score (Sec. 3.3 "Precision"; Alg. 1 step 3, one layer / KV head)
# --------------------------------------------------------------------------
def exact_scores(q_win, k_blk, k_ctx=None, block_pos0=0, q_pos0=None, causal=True, row_lse=None,
                 row_lse_complete=None):
    """S_exact[h, i] for every block key i of every KV head h.

    q_win [H_q, W, d]  window queries, query head h*G+g belongs to KV head h
    k_blk [H_kv, S_t, d] block keys, key i sits at position block_pos0 + i
    k_ctx [H_kv, T, d] or None: look-back keys, always visible, normaliser only
    q_pos0: position of window query 0 (default: window = last W block tokens)
    row_lse [H_q, W] or None: natural-log sum over keys OUTSIDE this call of exp(q . k / sqrt(d)) for
        every window query (what an attention kernel over the rest of the cache reports); those keys
        join the normaliser exactly as look-back keys do (Sec. 3.2 boundary smoothing, extended to
        context that is not re-read).

    row_lse_complete [H_q, W] or None: the COMPLETE natural-log normaliser of every window query, over all
        keys the row attends to, as the model's own attention reports it (Sec. 3.3 "Precision": the score is
        the attention the model computes).  Then p = exp(l - row_lse_complete) at the visible block keys;
        k_ctx and row_lse are not used.

    Row (g, j): logits l = q . k / sqrt(d) over the T + S_t keys, block key i
    masked when causal and block_pos0 + i > q_pos0 + j, p = softmax(l);
    S_exact[h, i] = (1 / (G W)) sum_g sum_j p[(g, j), T + i].
    """
    q_win = np.asarray(q_win, dtype=np.float64)
    k_blk = np.asarray(k_blk, dtype=np.float64)
    h_q, w, d = q_win.shape
    h_kv, s_t, d2 = k_blk.shape
    assert d == d2 and h_q % h_kv == 0
    g_sz = h_q // h_kv
    t_ctx = 0 if k_ctx is None else int(np.asarray(k_ctx).shape[1])
    if q_pos0 is None:
        q_pos0 = block_pos0 + s_t - w
    key_pos = block_pos0 + np.arange(s_t)
    qry_pos = q_pos0 + np.arange(w)
    visible = np.ones((w, s_t), dtype=bool)
    if causal:
        visible = key_pos[None, :] <= qry_pos[:, None]
    out = np.zeros((h_kv, s_t), dtype=np.float64)
    if row_lse_complete is not None:
        lse = np.asarray(row_lse_complete, dtype=np.float64)
        for h in range(h_kv):
            for g in range(g_sz):
                logits = (q_win[h * g_sz + g] @ k_blk[h].T) / np.sqrt(np.float64(d))
                p = np.where(visible, np.exp(logits - lse[h * g_sz + g][:, None]), 0.0)
                out[h] += p.sum(axis=0)
        return out / np.float64(g_sz * w)
    for h in range(h_kv):
        if t_ctx:
            keys = np.concatenate([np.asarray(k_ctx[h], dtype=np.float64), k_blk[h]], axis=0)
        else:
            keys = k_blk[h]
        vis = np.concatenate([np.ones((w, t_ctx), dtype=bool), visible], axis=1)
        for g in range(g_sz):
            logits = (q_win[h * g_sz + g] @ keys.T) / np.sqrt(np.float64(d))
            logits = np.where(vis, logits, -np.inf)
            row_max = logits.max(axis=1, keepdims=True)
            e = np.exp(logits - row_max)
            denom = e.sum(axis=1, keepdims=True)
            if row_lse is not None:
                ext = np.asarray(row_lse, dtype=np.float64)[h * g_sz + g][:, None]
                denom = denom + np.exp(ext - row_max)
            p = e / denom
            out[h] += p[:, t_ctx:].sum(axis=0)
    return out / np.float64(g_sz * w)


# --------------------------------------------------------------------------
# a2  SimHash signatures (Sec. 3.3 "Recall"; the hash functions h_r of Alg. 1)
# --------------------------------------------------------------------------
def simhash(x, planes, n_tables: int, n_bits: int):
    """Random-hyperplane codes of the vectors x[..., d].

    planes [n_tables * n_bits, d]; row r*n_bits + c is bit c of table r.
    bit = 1 when planes[row] . x >= 0; code = sum_c bit_c 2^c.
    Returns (sig [..., n_tables] int64, unsure [..., n_tables] bool) where
    unsure marks codes with a projection of magnitude below UNSURE_EPS.
    """
    x = np.asarray(x, dtype=np.float64)
    planes = np.asarray(planes, dtype=np.float64)
    assert planes.shape[0] == n_tables * n_bits
    proj = x @ planes.T                                   # [..., L*K]
    proj = proj.reshape(x.shape[:-1] + (n_tables, n_bits))
    bits = (proj >= 0.0).astype(np.int64)
    weights = (np.int64(1) << np.arange(n_bits, dtype=np.int64))
    sig = (bits * weights).sum(axis=-1)
    unsure = (np.abs(proj) < UNSURE_EPS).any(axis=-1)
    return sig, unsure


# --------------------------------------------------------------------------
# a3  collision counts (Alg. 1 step 6)
# --------------------------------------------------------------------------
def collision_counts(sig_q, sig_k, g_sz: int):
    """cnt[h, i] = sum_g sum_j sum_r [ sig_q[h*G+g, j, r] == sig_k[h, i, r] ].

    S_lsh = cnt / (G * W * R) is Alg. 1's indicator average; the integer count
    carries the same order and is what the selection ranks by.
    """
    sig_q = np.asarray(sig_q)
    sig_k = np.asarray(sig_k)
    h_q, w, n_tables = sig_q.shape
    h_kv, s_t, _ = sig_k.shape
    assert h_q == h_kv * g_sz
    cnt = np.zeros((h_kv, s_t), dtype=np.int64)
    for h in range(h_kv):
        codes_q = sig_q[h * g_sz:(h + 1) * g_sz].reshape(g_sz * w, n_tables)
        for r in range(n_tables):
            eq = codes_q[:, r][:, None] == sig_k[h, :, r][None, :]   # [G*W, S_t]
            cnt[h] += eq.sum(axis=0)
    return cnt


def lsh_scores(cnt, g_sz: int, w: int, n_tables: int):
    """S_lsh of Alg. 1 step 6: the collision indicators' average."""
    return np.asarray(cnt, dtype=np.float64) / np.float64(g_sz * w * n_tables)


# --------------------------------------------------------------------------
# a4  Exact-LSH selection (Alg. 1 steps 4-8 plus the Sec. 3.1 partition)
# --------------------------------------------------------------------------
def select(s_exact, cnt, n_anchor: int, n_local: int, k_exact: int, k_lsh: int):
    """Kept token indices of one head's block, ascending.

    Protected P = first n_anchor and last n_local positions (always kept).
    Candidates C = the rest.  K_exact = the k_exact candidates ranked first by
    (S_exact descending, index ascending); K_lsh = the k_lsh members of
    C minus K_exact ranked first by (cnt descending, index ascending).
    Returns (keep, K_exact, K_lsh) as sorted int64 arrays.
    """
    s_exact = np.asarray(s_exact, dtype=np.float64)
    cnt = np.asarray(cnt)
    s_t = s_exact.shape[0]
    if n_anchor + n_local > s_t:
        raise ValueError("protected sets exceed the block")
    cand = list(range(n_anchor, s_t - n_local))
    if k_exact + k_lsh > len(cand):
        raise ValueError("recall budget exceeds the candidate set")
    by_exact = sorted(cand, key=lambda i: (-s_exact[i], i))
    k_ex = by_exact[:k_exact]
    taken = set(k_ex)
    residual = [i for i in cand if i not in taken]
    by_lsh = sorted(residual, key=lambda i: (-int(cnt[i]), i))
    k_l = by_lsh[:k_lsh]
    protected = list(range(n_anchor)) + list(range(s_t - n_local, s_t))
    keep = sorted(set(protected) | taken | set(k_l))
    return (np.asarray(keep, dtype=np.int64),
            np.asarray(sorted(k_ex), dtype=np.int64),
            np.asarray(sorted(k_l), dtype=np.int64))


# --------------------------------------------------------------------------
# a5  append-only cache (Sec. 1 contribution 1; Sec. 3 first paragraph)
# --------------------------------------------------------------------------
def append(cache_k, cache_v, cache_pos, cache_len: int, k_blk, v_blk, keep, block_pos0: int):
    """Copy the kept rows of every head to the end of the cache, in place.

    cache_k / cache_v [H_kv, cap, d], cache_pos [H_kv, cap] absolute positions,
    keep [H_kv, B_t] ascending block-local indices.  Returns the new length.
    """
    keep = np.asarray(keep)
    h_kv, b_t = keep.shape
    if cache_len + b_t > cache_k.shape[1]:
        raise ValueError("cache capacity exceeded")
    for h in range(h_kv):
        cache_k[h, cache_len:cache_len + b_t] = k_blk[h, keep[h]]
        cache_v[h, cache_len:cache_len + b_t] = v_blk[h, keep[h]]
        cache_pos[h, cache_len:cache_len + b_t] = block_pos0 + keep[h]
    return cache_len + b_t


# --------------------------------------------------------------------------
# attention over the compacted cache (Sec. 3 first paragraph: the kept tokens
# are what later tokens attend to; Sec. 3.2 / 3.3: its row normaliser)
# --------------------------------------------------------------------------
def attend_cache(q, cache_k, cache_v, cache_len: int):
    """Softmax attention of every query over the first cache_len rows of its KV head's cache.

    q [H_q, n_q, d]; cache_k / cache_v [H_kv, cap, d]; query head h*G+g reads KV head h.  Every cached row
    is visible: the cache holds earlier blocks only (append-only, Sec. 1 contribution 1).

    Row (hq, j): l_i = q . k_i / sqrt(d) over i < cache_len, p = softmax(l), out = sum_i p_i v_i,
    lse = log sum_i exp(l_i) (natural logarithm).  Returns (out [H_q, n_q, d], lse [H_q, n_q]).
    With cache_len = 0 the output is zero and lse = -inf.  lse is what exact_scores takes as row_lse.
    """
    q = np.asarray(q, dtype=np.float64)
    h_q, n_q, d = q.shape
    h_kv = np.asarray(cache_k).shape[0]
    assert h_q % h_kv == 0
    g_sz = h_q // h_kv
    out = np.zeros((h_q, n_q, d), dtype=np.float64)
    lse = np.full((h_q, n_q), -np.inf, dtype=np.float64)
    if cache_len == 0:
        return out, lse
    for hq in range(h_q):
        keys = np.asarray(cache_k[hq // g_sz][:cache_len], dtype=np.float64)
        vals = np.asarray(cache_v[hq // g_sz][:cache_len], dtype=np.float64)
        logits = (q[hq] @ keys.T) / np.sqrt(np.float64(d))
        row_max = logits.max(axis=1, keepdims=True)
        e = np.exp(logits - row_max)
        denom = e.sum(axis=1, keepdims=True)
        out[hq] = (e / denom) @ vals
        lse[hq] = (row_max + np.log(denom))[:, 0]
    return out, lse


def attend_block(q, cache_k, cache_v, cache_len: int, k_blk, v_blk, block_pos0=0, q_pos0=None, causal=True):
    """The block's own prefill attention: every query over the compacted cache followed by the block's keys.

    q [H_q, n_q, d] are queries at absolute positions q_pos0 + j (default: the block's last n_q tokens);
    cache_k / cache_v [H_kv, cap, d], the first cache_len rows of which are earlier blocks' kept tokens, all
    visible (Sec. 3 first paragraph: only the kept tokens remain for later tokens to attend to); k_blk / v_blk
    [H_kv, S_t, d] the current block at absolute positions block_pos0 + i, key i visible to query j iff
    block_pos0 + i <= q_pos0 + j when causal.  One softmax per row over both segments:
    out = sum_i p_i v_i, lse = log sum_i exp(l_i) over the visible keys (natural logarithm).  For the window
    rows this lse is the complete normaliser of Alg. 1 step 3 (what exact_scores takes as row_lse_complete
    when the look-back keys are inside the cache).  A row that sees no key gives zero and -inf.
    Returns (out [H_q, n_q, d], lse [H_q, n_q]).
    """
    q = np.asarray(q, dtype=np.float64)
    h_q, n_q, d = q.shape
    k_blk = np.asarray(k_blk, dtype=np.float64)
    v_blk = np.asarray(v_blk, dtype=np.float64)
    h_kv, s_t, _ = k_blk.shape
    assert h_q % h_kv == 0
    g_sz = h_q // h_kv
    if q_pos0 is None:
        q_pos0 = block_pos0 + s_t - n_q
    out = np.zeros((h_q, n_q, d), dtype=np.float64)
    lse = np.full((h_q, n_q), -np.inf, dtype=np.float64)
    key_pos = block_pos0 + np.arange(s_t)
    for hq in range(h_q):
        h = hq // g_sz
        keys = np.concatenate([np.asarray(cache_k[h][:cache_len], dtype=np.float64).reshape(cache_len, d), k_blk[h]])
        vals = np.concatenate([np.asarray(cache_v[h][:cache_len], dtype=np.float64).reshape(cache_len, d), v_blk[h]])
        for j in range(n_q):
            visible = np.ones(cache_len + s_t, dtype=bool)
            if causal:
                visible[cache_len:] = key_pos <= q_pos0 + j
            if not visible.any():
                continue
            logits = (keys[visible] @ q[hq, j]) / np.sqrt(np.float64(d))
            top = logits.max()
            e = np.exp(logits - top)
            denom = e.sum()
            out[hq, j] = (e / denom) @ vals[visible]
            lse[hq, j] = top + np.log(denom)
    return out, lse


# --------------------------------------------------------------------------
# one block, one layer: the composition the C-ABI entry points implement
# --------------------------------------------------------------------------
def select_block(q_win, k_blk, k_ctx, planes, n_tables, n_bits,
                 n_anchor, n_local, k_exact, k_lsh,
                 block_pos0=0, q_pos0=None, causal=True, row_lse=None, row_lse_complete=None):
    """Steps a1-a4 for all KV heads of one block.  Returns a dict of every stage."""
    h_q = np.asarray(q_win).shape[0]
    h_kv = np.asarray(k_blk).shape[0]
    g_sz = h_q // h_kv
    s_ex = exact_scores(q_win, k_blk, k_ctx, block_pos0, q_pos0, causal, row_lse, row_lse_complete)
    sig_k, uns_k = simhash(k_blk, planes, n_tables, n_bits)
    sig_q, uns_q = simhash(q_win, planes, n_tables, n_bits)
    cnt = collision_counts(sig_q, sig_k, g_sz)
    keep, k_ex, k_l = [], [], []
    for h in range(h_kv):
        kp, ke, kl = select(s_ex[h], cnt[h], n_anchor, n_local, k_exact, k_lsh)
        keep.append(kp)
        k_ex.append(ke)
        k_l.append(kl)
    return dict(s_exact=s_ex, sig_k=sig_k, sig_q=sig_q, unsure_k=uns_k, unsure_q=uns_q,
                cnt=cnt, keep=np.stack(keep), k_exact_set=k_ex, k_lsh_set=k_l)


def consensus_block(layers, n_tables, n_bits, n_anchor, n_local, k_exact, k_lsh,
                    block_pos0=0, q_pos0=None, causal=True):
    """Alg. 1 steps 3-8 with the sum of step 3 taken over all layers and heads.

    layers: sequence of dicts, one per layer, with q_win [H_q, W, d], k_blk [H_kv, S_t, d],
    k_ctx [H_kv, T, d] or None, planes [L*K, d] (each layer may bring its own hyperplanes).
    The exact score of a token is the plain sum of the per-head pooled probabilities
    (Sec. 3.3 "Precision"; Alg. 1 step 3: the sum runs over every layer and head); its collision count is the
    plain sum of the per-head counts (Alg. 1 step 6 averages the same indicator over r; the
    sum over heads and layers keeps the order of that average).  One two-stage TopK (steps 4-8)
    on the summed arrays gives one kept set for every layer and head.

    Returns dict(score [S_t], count [S_t], keep [B_t], per_layer=[select_block-style stage dicts]).
    """
    score, count, stages = None, None, []
    for lay in layers:
        h_q = np.asarray(lay["q_win"]).shape[0]
        h_kv = np.asarray(lay["k_blk"]).shape[0]
        s_ex = exact_scores(lay["q_win"], lay["k_blk"], lay.get("k_ctx"), block_pos0, q_pos0, causal)
        sig_k, uns_k = simhash(lay["k_blk"], lay["planes"], n_tables, n_bits)
        sig_q, uns_q = simhash(lay["q_win"], lay["planes"], n_tables, n_bits)
        cnt = collision_counts(sig_q, sig_k, h_q // h_kv)
        stages.append(dict(s_exact=s_ex, sig_k=sig_k, sig_q=sig_q, unsure_k=uns_k, unsure_q=uns_q, cnt=cnt))
        for h in range(h_kv):
            score = s_ex[h].copy() if score is None else score + s_ex[h]
            count = cnt[h].copy() if count is None else count + cnt[h]
    keep, k_ex, k_l = select(score, count, n_anchor, n_local, k_exact, k_lsh)
    return dict(score=score, count=count, keep=keep, k_exact_set=k_ex, k_lsh_set=k_l, per_layer=stages)


def compress_layer(blocks, planes, n_tables, n_bits, B, n, alpha, cap, dtype=np.float64):
    """Run a whole layer: blocks is an iterable of (q_win, k_blk, v_blk, block_pos0).

    Look-back (Sec. 3.2): block t's scoring sees, as context-only keys, the
    previous block's local window, i.e. the last n_local cache rows.
    Returns (cache_k, cache_v, cache_pos, cache_len, per-block stage dicts).
    """
    cache_k = cache_v = cache_pos = None
    cache_len = 0
    prev_local = 0
    stages = []
    for (q_win, k_blk, v_blk, pos0) in blocks:
        k_blk = np.asarray(k_blk, dtype=np.float64)
        v_blk = np.asarray(v_blk, dtype=np.float64)
        h_kv, s_t, d = k_blk.shape
        if cache_k is None:
            cache_k = np.zeros((h_kv, cap, d), dtype=dtype)
            cache_v = np.zeros((h_kv, cap, d), dtype=dtype)
            cache_pos = np.full((h_kv, cap), -1, dtype=np.int64)
        na, nl, ke, kl = partition(B, n, alpha, s_t)
        k_ctx = None
        if cache_len and prev_local:
            k_ctx = cache_k[:, cache_len - prev_local:cache_len].astype(np.float64)
        st = select_block(q_win, k_blk, k_ctx, planes, n_tables, n_bits,
                          na, nl, ke, kl, block_pos0=pos0)
        cache_len = append(cache_k, cache_v, cache_pos, cache_len, k_blk, v_blk, st["keep"], pos0)
        prev_local = nl
        stages.append(st)
    return cache_k, cache_v, cache_pos, cache_len, stages


def compress_layer_deferred(blocks, planes, n_tables, n_bits, B, n, alpha, cap, tail, dtype=np.float64):
    """The layer loop with the look-back of Sec. 3.2 read as DEFERRING a block's edge: the last `tail`
    tokens of block t are not judged with block t (no later context has been seen for them) but join the
    candidates of block t+1; the last block defers nothing, so every token is judged exactly once.

    Segment t = [deferred tail of block t-1 | block t without its own tail], scored by block t's
    observation window (its last W tokens, at their real positions: the window then reaches `tail`
    tokens past the segment's end, and the causal mask follows positions).  Everything else is
    compress_layer applied to the segments: budget B per segment (B_t = min(B, segment length)), the
    Sec. 3.1 partition on the segment, and the previous SEGMENT's local window (the cache's last n_local
    rows, the tokens just before the segment) as context-only keys.  tail = 0 is compress_layer.

    blocks: iterable of (q_win, k_blk, v_blk, block_pos0), consecutive in position.
    Returns (cache_k, cache_v, cache_pos, cache_len, per-segment stage dicts); each stage dict also
    carries seg_pos0 and seg_len.
    """
    blocks = list(blocks)
    cache_k = cache_v = cache_pos = None
    cache_len = 0
    prev_local = 0
    pend_k = pend_v = None
    stages = []
    for t, (q_win, k_blk, v_blk, pos0) in enumerate(blocks):
        k_blk = np.asarray(k_blk, dtype=np.float64)
        v_blk = np.asarray(v_blk, dtype=np.float64)
        h_kv, s_t, d = k_blk.shape
        w = np.asarray(q_win).shape[1]
        tail_t = 0 if t == len(blocks) - 1 else int(tail)
        if tail_t > s_t:
            raise ValueError("tail longer than a block")
        if cache_k is None:
            cache_k = np.zeros((h_kv, cap, d), dtype=dtype)
            cache_v = np.zeros((h_kv, cap, d), dtype=dtype)
            cache_pos = np.full((h_kv, cap), -1, dtype=np.int64)
        n_pend = 0 if pend_k is None else pend_k.shape[1]
        seg_k = k_blk[:, :s_t - tail_t] if n_pend == 0 else np.concatenate([pend_k, k_blk[:, :s_t - tail_t]], axis=1)
        seg_v = v_blk[:, :s_t - tail_t] if n_pend == 0 else np.concatenate([pend_v, v_blk[:, :s_t - tail_t]], axis=1)
        pend_k = k_blk[:, s_t - tail_t:] if tail_t else None
        pend_v = v_blk[:, s_t - tail_t:] if tail_t else None
        seg_pos0 = pos0 - n_pend
        seg_len = seg_k.shape[1]
        na, nl, ke, kl = partition(B, n, alpha, seg_len)
        k_ctx = None
        if cache_len and prev_local:
            k_ctx = cache_k[:, cache_len - prev_local:cache_len].astype(np.float64)
        st = select_block(q_win, seg_k, k_ctx, planes, n_tables, n_bits, na, nl, ke, kl,
                          block_pos0=seg_pos0, q_pos0=pos0 + s_t - w)
        cache_len = append(cache_k, cache_v, cache_pos, cache_len, seg_k, seg_v, st["keep"], seg_pos0)
        prev_local = nl
        st["seg_pos0"], st["seg_len"] = seg_pos0, seg_len
        stages.append(st)
    return cache_k, cache_v, cache_pos, cache_len, stages
