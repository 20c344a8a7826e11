"""GPU parity of the global-consensus variant (laserkv_score_block / laserkv_select_consensus /
laserkv_append_shared) against the oracle's consensus_block on the same seeded inputs."""
import sys

import numpy as np
import pytest
import torch

from oracle import laserkv_oracle as O
from paper_2602_02199_amd import binding, synth
from tests.parity_util import TOL, count_interval

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


@pytest.mark.parametrize("name,n_layers,n_blocks,kw", [
    ("tiny", 3, 3, dict()),
    ("llama8b-16k", 2, 2, dict(l_ctx=4096)),
    ("tiny", 2, 2, dict(lsh_tables=3, lsh_bits=16, l_ctx=1024)),     # wide codes: the stand-alone count kernel
])
def test_consensus_matches_oracle(name, n_layers, n_blocks, kw):
    wl = synth.shrink(synth.WORKLOADS[name], index=20, **kw)
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    parts = O.partition(B, wl.n_div, wl.alpha, wl.s_block)
    na, nl, ke, kl = parts
    b_t = sum(parts)
    s = wl.s_block
    tol = TOL[wl.dtype]
    data = [synth.make_layer(wl, layer, na, n_blocks=n_blocks) for layer in range(n_layers)]
    dev = [{k: v.to(DEV) for k, v in d.items() if k != "needles"} for d in data]
    lib = binding.LaserKV(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.dtype, wl.lsh_tables, wl.lsh_bits,
                          max_block=s, max_window=wl.window, max_ctx_keys=nl)
    cap = n_blocks * b_t
    caches = [dict(k=torch.zeros(wl.n_kv_heads, cap, wl.head_dim, dtype=wl.torch_dtype, device=DEV),
                   v=torch.zeros(wl.n_kv_heads, cap, wl.head_dim, dtype=wl.torch_dtype, device=DEV),
                   pos=torch.full((wl.n_kv_heads, cap), -1, dtype=torch.int64, device=DEV)) for _ in range(n_layers)]
    score = torch.empty(s, dtype=torch.float32, device=DEV)
    count = torch.empty(s, dtype=torch.int32, device=DEV)
    results = []
    cache_len = 0
    for t in range(n_blocks):
        lo = t * s
        n_ctx = nl if t else 0
        for li in range(n_layers):
            k_ctx = caches[li]["k"][:, cache_len - n_ctx:cache_len] if n_ctx else None
            lib.laserkv_score_block(dev[li]["q_win"][t], dev[li]["k"][:, lo:lo + s], k_ctx, dev[li]["planes"],
                                    block_pos0=lo, score_acc=score, count_acc=count, accumulate=li > 0)
        keep = torch.empty(b_t, dtype=torch.int32, device=DEV)
        lib.laserkv_select_consensus(score, count, s_t=s, n_anchor=na, n_local=nl, k_exact=ke, k_lsh=kl, keep_idx=keep)
        for li in range(n_layers):
            lib.laserkv_append_shared(dev[li]["k"][:, lo:lo + s], dev[li]["v"][:, lo:lo + s], keep, b_t=b_t,
                                      block_pos0=lo, k_cache=caches[li]["k"], v_cache=caches[li]["v"],
                                      cache_pos=caches[li]["pos"], cache_len=cache_len)
        cache_len += b_t
        torch.cuda.synchronize()
        results.append((score.cpu().numpy().astype(np.float64), count.cpu().numpy().astype(np.int64),
                        keep.cpu().numpy().astype(np.int64)))
    g = wl.group
    for t, (g_score, g_count, g_keep) in enumerate(results):
        lo = t * s
        n_ctx = nl if t else 0
        layers = [dict(q_win=f64(d["q_win"][t]), k_blk=f64(d["k"][:, lo:lo + s]),
                       k_ctx=f64(d["k"][:, lo - n_ctx:lo]) if n_ctx else None, planes=f64(d["planes"])) for d in data]
        c = O.consensus_block(layers, wl.lsh_tables, wl.lsh_bits, *parts, block_pos0=lo)
        cand = np.arange(na, s - nl)
        s_k = np.sort(c["score"][cand])[::-1][ke - 1] if ke else 0.0
        err = np.abs(g_score - c["score"])
        assert np.all(err <= tol * c["score"] + tol * s_k), f"block {t}: summed score off by {float(err.max()):.3e}"
        c_lo = np.zeros(s, dtype=np.int64)
        c_hi = np.zeros(s, dtype=np.int64)
        unsure = 0
        for stg in c["per_layer"]:
            a, b = count_interval(stg["sig_q"], stg["sig_k"], stg["unsure_q"], stg["unsure_k"], g)
            c_lo += a.sum(0)
            c_hi += b.sum(0)
            unsure += int(stg["unsure_q"].sum() + stg["unsure_k"].sum())
        assert np.all((c_lo <= g_count) & (g_count <= c_hi)), f"block {t}: summed count outside its interval"
        if not unsure:
            assert np.array_equal(g_count, c["count"])
        own, _, _ = O.select(g_score, g_count, *parts)
        assert np.array_equal(g_keep, own), "kept set is not Alg. 1 applied to the path's own sums"
        diff = np.setxor1d(g_keep, c["keep"])
        if diff.size:
            resid = np.setdiff1d(cand, c["k_exact_set"])
            c_k = np.sort(c["count"][resid])[::-1][kl - 1] if kl else None
            for i in diff:
                near_s = abs(c["score"][i] - s_k) <= tol * s_k
                near_c = c_k is not None and c_lo[i] <= c_k <= c_hi[i]
                assert near_s or near_c, f"block {t} token {i}: kept sets differ beyond tolerance"
        print(f"[consensus {wl.name} blk {t}] unsure codes {unsure}, max score err/(s+s_k) "
              f"{float((err / (c['score'] + s_k)).max()):.2e}, tolerated index diffs {diff.size}", flush=True)
        sys.stdout.flush()
        # every layer and head appended exactly the shared rows
        pos = torch.from_numpy(g_keep + lo).to(DEV)
        for li in range(n_layers):
            sl = slice(t * b_t, (t + 1) * b_t)
            assert torch.equal(caches[li]["pos"][:, sl], pos.expand(wl.n_kv_heads, -1))
            assert torch.equal(caches[li]["k"][:, sl], dev[li]["k"][:, pos])
            assert torch.equal(caches[li]["v"][:, sl], dev[li]["v"][:, pos])
    for li in range(n_layers):
        assert bool((caches[li]["pos"][:, cache_len:] == -1).all())


def test_consensus_error_paths():
    wl = synth.WORKLOADS["tiny"]
    lib = binding.LaserKV(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.dtype, wl.lsh_tables, wl.lsh_bits,
                          max_block=512, max_window=32, max_ctx_keys=64)
    score = torch.zeros(512, dtype=torch.float32, device=DEV)
    count = torch.zeros(512, dtype=torch.int32, device=DEV)
    keep = torch.full((100,), -7, dtype=torch.int32, device=DEV)
    with pytest.raises(binding.LaserKVError):     # recall budget larger than the candidate set
        lib.laserkv_select_consensus(score, count, s_t=512, n_anchor=200, n_local=200, k_exact=100, k_lsh=100, keep_idx=keep)
    with pytest.raises(binding.LaserKVError):     # block longer than the context allows
        lib.laserkv_select_consensus(score, count, s_t=513, n_anchor=1, n_local=1, k_exact=1, k_lsh=1, keep_idx=keep)
    torch.cuda.synchronize()
    assert bool((keep == -7).all())
