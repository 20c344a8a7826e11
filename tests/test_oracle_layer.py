"""The oracle's block loop on the tiny workload: invariants of the accumulative, append-only policy
(Sec. 1 contribution 1; Sec. 3; Sec. 3.2 look-back) and a sanity check that planted needles survive."""
import numpy as np
import torch

from oracle import laserkv_oracle as O
from paper_2602_02199_amd import synth


def test_generator_is_deterministic_and_needles_align():
    wl = synth.WORKLOADS["tiny"]
    a = synth.make_layer(wl, 0, 56, n_blocks=2)
    b = synth.make_layer(wl, 0, 56, n_blocks=2)
    full = synth.make_layer(wl, 0, 56, n_blocks=3)
    for key in ("planes", "q_win", "k", "v", "needles"):
        assert torch.equal(a[key], b[key])
    assert torch.equal(full["k"][:, : 2 * wl.s_block], a["k"])           # a prefix of the longer run
    other = synth.make_layer(wl, 1, 56, n_blocks=1)
    assert not torch.equal(other["k"], a["k"][:, : wl.s_block])
    assert a["needles"].shape == (2 * wl.n_kv_heads * wl.needles_per_block, 3)
    g = wl.group
    for blk, h, p in a["needles"].tolist():
        assert 56 <= p < wl.s_block - 56
        key = a["k"][h, blk * wl.s_block + p].double()
        qs = a["q_win"][blk, h * g:(h + 1) * g].reshape(-1, wl.head_dim).double()
        cos = (qs @ key) / (qs.norm(dim=1) * key.norm())
        assert abs(cos.max().item() - 0.9) < 1e-4


def test_layer_run_invariants_tiny():
    wl = synth.WORKLOADS["tiny"]
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    assert B == 227
    na, nl, ke, kl = O.partition(B, wl.n_div, wl.alpha, wl.s_block)
    n_blocks = 4
    data = synth.make_layer(wl, 0, na, n_blocks=n_blocks)
    k = data["k"].double().numpy(); v = data["v"].double().numpy(); q = data["q_win"].double().numpy()
    blocks = [(q[t], k[:, t * wl.s_block:(t + 1) * wl.s_block], v[:, t * wl.s_block:(t + 1) * wl.s_block], t * wl.s_block)
              for t in range(n_blocks)]
    ck, cv, cp, length, stages = O.compress_layer(blocks, data["planes"].double().numpy(), wl.lsh_tables, wl.lsh_bits,
                                                  B, wl.n_div, wl.alpha, cap=n_blocks * B)
    assert length == n_blocks * B                                        # accumulative: exactly B per block
    assert np.all(np.diff(cp[:, :length], axis=1) > 0)                    # append-only ordering
    for h in range(wl.n_kv_heads):
        assert np.array_equal(ck[h, :length], k[h, cp[h, :length]])      # rows are verbatim copies
        assert np.array_equal(cv[h, :length], v[h, cp[h, :length]])
    for t, st in enumerate(stages):
        assert st["keep"].shape == (wl.n_kv_heads, B)
        assert np.allclose(st["s_exact"].sum(1) <= 1.0 + 1e-12, True)
        if t == 0:
            np.testing.assert_allclose(st["s_exact"].sum(1), 1.0, atol=1e-12)   # no look-back in block 0
        else:
            assert np.all(st["s_exact"].sum(1) < 1.0)                            # look-back keys took mass
        assert st["cnt"].max() <= wl.group * wl.window * wl.lsh_tables
    kept = {(t, h, int(p)) for t, st in enumerate(stages) for h in range(wl.n_kv_heads) for p in st["keep"][h]}
    for blk, h, p in data["needles"].tolist():
        assert (blk, h, p) in kept                                        # sanity: needles are heavy hitters


def test_tiny_kept_sets_match_the_stored_run():
    """The oracle and the seeded generator still produce the kept sets stored by
    tests/golden/make_tiny_keep.py (a drift guard, not an independent pin)."""
    import importlib.util
    import os
    here = os.path.dirname(os.path.abspath(__file__))
    spec = importlib.util.spec_from_file_location("make_tiny_keep", os.path.join(here, "golden", "make_tiny_keep.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    stored = [ln.strip() for ln in open(os.path.join(here, "golden", "tiny_keep_sets.txt")) if ln.strip() and not ln.startswith("#")]
    assert mod.compute() == stored
