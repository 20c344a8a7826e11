"""GPU parity of laserkv_attend_block (the block's own prefill attention over the compacted cache followed by
the block's keys under the causal mask; Sec. 3 first paragraph, Sec. 3.3 "Precision") against the oracle,
element by element through the C-ABI, and its use as the source of the complete row statistics of the
selection (laserkv_set_row_lse_complete).

Comparison rule as for laserkv_attend_cache: |gpu - oracle| <= tol * (|oracle| + sum_i p_i |v_i|) per output
element (bf16 2e-2 with a regression bound of 3e-3 on what is observed, fp32 1e-5), log-sum-exp within 1e-4.
"""
import numpy as np
import pytest
import torch

from oracle import laserkv_oracle as O
from paper_2602_02199_amd import binding, synth
from tests.parity_util import check_block
from tests.test_gpu_attend import DEV, OBSERVED, TOL, f64, make_inputs, say

pytestmark = pytest.mark.gpu


def run_block(lib, q, kc, vc, n, kb, vb, block_pos0, q_pos0, causal=True):
    out = torch.full(q.shape, float("nan"), dtype=torch.float32, device=DEV)
    lse = torch.full(q.shape[:2], float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.empty(lib.laserkv_attend_block_workspace_bytes(q.shape[1], n, kb.shape[1]), dtype=torch.uint8, device=DEV)
    lib.laserkv_attend_block(q, kc, vc, kb, vb, cache_len=n, block_pos0=block_pos0, q_pos0=q_pos0, causal=causal,
                             out=out, out_lse=lse, workspace=ws)
    torch.cuda.synchronize()
    return out.cpu().numpy(), lse.cpu().numpy()


def compare_block(out, lse, q, kc, vc, n, kb, vb, block_pos0, q_pos0, causal, dtype, label):
    args = dict(block_pos0=block_pos0, q_pos0=q_pos0, causal=causal)
    o_out, o_lse = O.attend_block(f64(q), f64(kc), f64(vc), n, f64(kb), f64(vb), **args)
    scale, _ = O.attend_block(f64(q), f64(kc), np.abs(f64(vc)), n, f64(kb), np.abs(f64(vb)), **args)
    blind = np.isneginf(o_lse)               # rows that see no key at all
    assert np.array_equal(np.isneginf(lse), blind), f"{label}: rows without a visible key differ"
    assert not out[blind].any()
    err = np.abs(out.astype(np.float64) - o_out)
    bound = TOL[dtype] * (np.abs(o_out) + scale)
    assert np.isfinite(out).all() and np.all(err <= bound), f"{label}: output off by up to {float((err - bound).max()):.3e} beyond tolerance"
    rel = float((err / (np.abs(o_out) + scale + 1e-300)).max())
    assert rel <= OBSERVED[dtype], f"{label}: output error {rel:.2e} exceeds the regression bound"
    dl = float(np.abs(lse.astype(np.float64)[~blind] - o_lse[~blind]).max()) if (~blind).any() else 0.0
    assert dl <= 1e-4, f"{label}: log-sum-exp off by {dl:.3e}"
    say(f"[attend_block {label}] max err/(|o|+scale) {rel:.2e}, max |lse diff| {dl:.2e}, blind rows {int(blind.sum())}")


CASES = [
    # label, dtype, H_q, H_kv, d, n_q, cache_len, s_t, q_pos0 - block_pos0 (None: the block's last n_q rows), causal
    ("tiny-whole-block", "f32", 4, 2, 64, 512, 454, 512, None, True),
    ("tiny-window-rows", "f32", 4, 2, 64, 32, 681, 512, None, True),
    ("f32-d128-ragged", "f32", 8, 2, 128, 70, 100, 70, None, True),
    ("bf16-whole-block-ragged", "bf16", 16, 4, 128, 600, 910, 600, None, True),
    ("bf16-window-rows", "bf16", 32, 8, 128, 64, 1820, 2048, None, True),
    ("bf16-no-cache", "bf16", 8, 2, 128, 300, 0, 300, None, True),
    ("bf16-no-mask", "bf16", 8, 4, 128, 40, 333, 500, 0, False),
    ("bf16-rows-before-the-block", "bf16", 8, 2, 64, 96, 200, 256, -40, True),
    ("bf16-rows-before-the-block-no-cache", "bf16", 4, 2, 64, 64, 0, 128, -10, True),
    ("bf16-decode-with-block", "bf16", 32, 8, 128, 1, 5000, 777, None, True),
    ("bf16-gqa8-two-row-groups", "bf16", 64, 8, 128, 64, 2049, 1000, None, True),
    ("f32-no-block", "f32", 4, 2, 64, 8, 300, 0, 0, True),
    ("bf16-d64-mid-block-rows", "bf16", 6, 2, 64, 100, 512, 1024, 300, True),
]


@pytest.mark.parametrize("case", CASES, ids=[c[0] for c in CASES])
def test_attend_block_against_oracle(case):
    label, dtype, h_q, h_kv, d, n_q, n, s_t, off, causal = case
    say(f"[attend_block {label}] {dtype} heads {h_q}/{h_kv} d {d} n_q {n_q} cache_len {n} s_t {s_t} offset {off}")
    cap = n + 70
    q, kk, vv = make_inputs(h_q, h_kv, d, n_q, cap + max(s_t, 1), dtype, seed=2000 + len(label))
    kc, vc = kk[:, :cap].clone(), vv[:, :cap].clone()
    kb, vb = kk[:, cap:cap + s_t].clone(), vv[:, cap:cap + s_t].clone()
    kc[:, n:] = float("nan")   # rows past cache_len must never be read
    vc[:, n:] = float("nan")
    block_pos0 = 4096
    q_pos0 = block_pos0 + (s_t - n_q if off is None else off)
    lib = binding.LaserKV(h_q, h_kv, d, dtype, 8, 8, max_block=max(s_t, n_q, 32), max_window=32, max_ctx_keys=0)
    out, lse = run_block(lib, q.to(DEV), kc.to(DEV), vc.to(DEV), n, kb.to(DEV), vb.to(DEV), block_pos0, q_pos0, causal)
    compare_block(out, lse, q, kc, vc, n, kb, vb, block_pos0, q_pos0, causal, dtype, label)
    lib.close()


def test_attend_block_strided_block_tensors_and_repeat():
    """K and V of the block taken as views of one fused [H_kv, S, 2, d] projection buffer (token stride 2 d) and
    queries from a wider buffer; hidden keys hold NaN-free garbage that must not weigh in; two runs are
    bit-identical; the result equals the one from contiguous copies."""
    h_q, h_kv, d, n_q, n, s_t = 16, 4, 128, 200, 700, 333
    q, kk, vv = make_inputs(h_q, h_kv, d, n_q, n + s_t, "bf16", seed=55)
    kc, vc, kb, vb = kk[:, :n].contiguous(), vv[:, :n].contiguous(), kk[:, n:].contiguous(), vv[:, n:].contiguous()
    fused = torch.zeros(h_kv, s_t + 5, 2, d, dtype=torch.bfloat16, device=DEV)
    fused[:, 2:2 + s_t, 0] = kb.to(DEV)
    fused[:, 2:2 + s_t, 1] = vb.to(DEV)
    kview, vview = fused[:, 2:2 + s_t, 0], fused[:, 2:2 + s_t, 1]
    wide = torch.zeros(h_q, n_q + 3, d + 64, dtype=torch.bfloat16, device=DEV)
    wide[:, 1:1 + n_q, :d] = q.to(DEV)
    lib = binding.LaserKV(h_q, h_kv, d, "bf16", 8, 8, max_block=512, max_window=32, max_ctx_keys=0)
    bp, qp = 1000, 1000 + s_t - n_q
    a = run_block(lib, wide[:, 1:1 + n_q, :d], kc.to(DEV), vc.to(DEV), n, kview, vview, bp, qp)
    b = run_block(lib, wide[:, 1:1 + n_q, :d], kc.to(DEV), vc.to(DEV), n, kview, vview, bp, qp)
    c = run_block(lib, q.to(DEV), kc.to(DEV), vc.to(DEV), n, kb.to(DEV), vb.to(DEV), bp, qp)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert np.array_equal(a[0], c[0]) and np.array_equal(a[1], c[1])
    compare_block(a[0], a[1], q, kc, vc, n, kb, vb, bp, qp, True, "bf16", "strided")
    lib.close()


def test_attend_block_without_block_keys_is_attend_cache():
    h_q, h_kv, d, n_q, n = 8, 2, 128, 16, 900
    q, k, v = (t.to(DEV) for t in make_inputs(h_q, h_kv, d, n_q, n, "bf16", seed=8))
    lib = binding.LaserKV(h_q, h_kv, d, "bf16", 8, 8, max_block=256, max_window=16, max_ctx_keys=0)
    a = run_block(lib, q, k, v, n, k[:, :0], v[:, :0], 0, 0)
    out = torch.empty(h_q, n_q, d, dtype=torch.float32, device=DEV)
    lse = torch.empty(h_q, n_q, dtype=torch.float32, device=DEV)
    ws = torch.empty(lib.laserkv_attend_workspace_bytes(n_q, n), dtype=torch.uint8, device=DEV)
    lib.laserkv_attend_cache(q, k, v, cache_len=n, out=out, out_lse=lse, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(a[0], out.cpu().numpy()) and np.array_equal(a[1], lse.cpu().numpy())
    lib.close()


def test_attend_block_error_paths():
    lib = binding.LaserKV(8, 2, 128, "bf16", 8, 8, max_block=64, max_window=16, max_ctx_keys=0)
    q, kk, vv = (t.to(DEV) for t in make_inputs(8, 2, 128, 64, 128, "bf16", seed=3))
    kc, vc, kb, vb = kk[:, :64].contiguous(), vv[:, :64].contiguous(), kk[:, 64:].contiguous(), vv[:, 64:].contiguous()
    out = torch.zeros(8, 64, 128, dtype=torch.float32, device=DEV)
    lse = torch.zeros(8, 64, dtype=torch.float32, device=DEV)
    ws = torch.empty(lib.laserkv_attend_block_workspace_bytes(64, 64, 64), dtype=torch.uint8, device=DEV)
    args = dict(cache_len=64, block_pos0=0, out=out, out_lse=lse)
    with pytest.raises(binding.LaserKVError) as e:
        lib.laserkv_attend_block(q, kc, vc, kb, vb, workspace=ws[:128], **args)
    assert e.value.code == binding.LKV_EINVAL and "workspace" in str(e.value)
    with pytest.raises(binding.LaserKVError):
        lib.laserkv_attend_block_workspace_bytes(65, 64, 64)                    # n_q > max_block
    with pytest.raises(binding.LaserKVError):
        lib.laserkv_attend_block_workspace_bytes(64, 64, 65)                    # s_t > max_block
    odd = torch.zeros(2, 64, 132, dtype=torch.bfloat16, device=DEV)            # token stride 264 bytes: rows not 16-byte aligned
    with pytest.raises(binding.LaserKVError) as e:
        lib.laserkv_attend_block(q, kc, vc, odd[:, :, :128], vb, workspace=ws, **args)
    assert "stride" in str(e.value)
    with pytest.raises(binding.LaserKVError):
        lib.laserkv_attend_block(q, None, None, kb, vb, workspace=ws, **args)   # cache_len > 0 without a cache
    torch.cuda.synchronize()
    assert not out.any() and not lse.any(), "a rejected call must launch nothing"
    lib.close()


@pytest.mark.parametrize("name,kw,whole", [("tiny", dict(l_ctx=2048), True), ("llama8b-16k", dict(l_ctx=8192), False)])
def test_complete_statistics_from_the_block_attention_kernel(name, kw, whole):
    """A layer run the way a model runs it: each block first attends to the compacted cache and, causally, to
    itself (laserkv_attend_block); the window rows' log-sum-exp that kernel reports is handed to the selection
    as the complete row statistic (laserkv_set_row_lse_complete), which then takes its single sweep; the kept
    rows join the cache the next block attends to.  `whole`: the attention call covers every row of the block
    (the model's call) and the window rows are copied out of its log-sum-exp; otherwise it covers the window
    rows only.  The oracle does the same with its own attention over its own cache."""
    wl = synth.shrink(synth.WORKLOADS[name], index=37, **kw)
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    parts = O.partition(B, wl.n_div, wl.alpha, wl.s_block)
    data = synth.make_layer(wl, 0, parts[0])
    nb, s, d, w = wl.n_blocks, wl.s_block, wl.head_dim, wl.window
    cap = nb * B
    td = wl.torch_dtype
    lib = binding.LaserKV(wl.n_q_heads, wl.n_kv_heads, d, wl.dtype, wl.lsh_tables, wl.lsh_bits,
                          max_block=s, max_window=w, max_ctx_keys=0)
    lib.laserkv_profile_begin()
    kc = torch.zeros(wl.n_kv_heads, cap, d, dtype=td, device=DEV)
    vc = torch.zeros_like(kc)
    pc = torch.zeros(wl.n_kv_heads, cap, dtype=torch.int64, device=DEV)
    ok = np.zeros((wl.n_kv_heads, cap, d)); ov = np.zeros_like(ok); op = np.zeros((wl.n_kv_heads, cap), dtype=np.int64)
    planes = data["planes"].to(DEV)
    gen = torch.Generator().manual_seed(5)
    length = 0
    for t in range(nb):
        lo = t * s
        q_win = data["q_win"][t]
        kb_h, vb_h = data["k"][:, lo:lo + s], data["v"][:, lo:lo + s]
        # the block's queries: random rows, the last w of them the observation window
        q_rows = torch.cat([torch.randn(wl.n_q_heads, s - w, d, generator=gen).to(td), q_win], dim=1) if whole else q_win
        n_q = q_rows.shape[1]
        q_dev, kb, vb = q_rows.to(DEV), kb_h.to(DEV), vb_h.to(DEV)
        out = torch.empty(wl.n_q_heads, n_q, d, dtype=torch.float32, device=DEV)
        lse = torch.empty(wl.n_q_heads, n_q, dtype=torch.float32, device=DEV)
        ws = torch.empty(lib.laserkv_attend_block_workspace_bytes(n_q, length, s), dtype=torch.uint8, device=DEV)
        lib.laserkv_attend_block(q_dev, kc, vc, kb, vb, cache_len=length, block_pos0=lo, out=out, out_lse=lse, workspace=ws)
        lse_win = lse[:, n_q - w:].contiguous()
        lib.laserkv_set_row_lse_complete(lse_win)
        dbg = dict(
            s_exact=torch.empty(wl.n_kv_heads, s, dtype=torch.float32, device=DEV),
            sig_k=torch.empty(wl.n_kv_heads, s, wl.lsh_tables, dtype=torch.int16, device=DEV),
            sig_q=torch.empty(wl.n_q_heads, w, wl.lsh_tables, dtype=torch.int16, device=DEV),
            cnt=torch.empty(wl.n_kv_heads, s, dtype=torch.int32, device=DEV))
        keep = torch.empty(wl.n_kv_heads, B, dtype=torch.int32, device=DEV)
        lib.laserkv_select_block(q_dev[:, n_q - w:], kb, None, planes, block_pos0=lo, n_anchor=parts[0], n_local=parts[1],
                                 k_exact=parts[2], k_lsh=parts[3], keep_idx=keep, dbg_s_exact=dbg["s_exact"],
                                 dbg_sig_k=dbg["sig_k"], dbg_sig_q=dbg["sig_q"], dbg_count=dbg["cnt"])
        lib.laserkv_append(kb, vb, keep, b_t=B, block_pos0=lo, k_cache=kc, v_cache=vc, cache_pos=pc, cache_len=length)
        torch.cuda.synchronize()
        # oracle: the same steps on its own cache
        compare_block(out.cpu().numpy(), lse.cpu().numpy(), q_rows, torch.from_numpy(ok), torch.from_numpy(ov), length,
                      kb_h, vb_h, lo, lo + s - n_q, True, wl.dtype, f"{wl.name} block {t}")
        _, o_lse = O.attend_block(f64(q_win), ok, ov, length, f64(kb_h), f64(vb_h), block_pos0=lo)
        st = O.select_block(f64(q_win), f64(kb_h), None, f64(data["planes"]), wl.lsh_tables, wl.lsh_bits, *parts,
                            block_pos0=lo, row_lse_complete=o_lse)
        g = dict(s_exact=dbg["s_exact"].cpu().numpy(), sig_k=dbg["sig_k"].cpu().numpy().view(np.uint16),
                 sig_q=dbg["sig_q"].cpu().numpy().view(np.uint16), cnt=dbg["cnt"].cpu().numpy(), keep=keep.cpu().numpy())
        rep = check_block(st, g, parts, wl.dtype)
        say(f"[attend_block->complete lse {wl.name} block {t}] score err {rep['max_rel']:.2e}, tolerated {rep['tolerated']}, "
            f"mass on block keys {float(st['s_exact'].sum(axis=1).mean()):.3f}")
        assert np.array_equal(g["keep"], st["keep"]), "kept sets differ by a threshold token: the caches diverge"
        O.append(ok, ov, op, length, f64(kb_h), f64(vb_h), st["keep"], lo)
        length += B
        if t:
            assert st["s_exact"].sum(axis=1).max() < 1.0 - 1e-6   # the cache took a share of the mass
    launches = {k: v[1] for k, v in lib.laserkv_profile_end().items()}
    assert launches["single"] == nb and launches["sweep1"] == 0 and launches["attend"] == nb
    assert np.array_equal(pc.cpu().numpy(), op)
    lib.laserkv_set_row_lse_complete(None)
    lib.close()


def test_attend_block_at_the_benchmark_size_on_sampled_rows():
    """The last block of the 128k workload in the launch shape bench.py times (4096 rows per query head over
    61 535 cache rows and the block's 4096 keys, one workgroup per 256 rows seeing all keys, direct output):
    sampled query positions (block start and end, row-tile and row-group edges, others) are recomputed one by
    one by the oracle for every head."""
    wl = synth.WORKLOADS["llama8b-128k"]
    h_q, h_kv, d, s = wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.s_block
    B = O.budget(s, wl.l_ctx, wl.r_num, wl.r_den)
    n = (wl.n_blocks - 1) * B
    q, kk, vv = make_inputs(h_q, h_kv, d, s, n + s, "bf16", seed=4242)
    kc, vc, kb, vb = kk[:, :n].contiguous(), vv[:, :n].contiguous(), kk[:, n:].contiguous(), vv[:, n:].contiguous()
    lib = binding.LaserKV(h_q, h_kv, d, "bf16", wl.lsh_tables, wl.lsh_bits, max_block=s, max_window=wl.window, max_ctx_keys=0)
    assert lib.laserkv_attend_block_workspace_bytes(s, n, s) == 256   # the direct route
    block_pos0 = (wl.n_blocks - 1) * s
    out, lse = run_block(lib, q.to(DEV), kc.to(DEV), vc.to(DEV), n, kb.to(DEV), vb.to(DEV), block_pos0, block_pos0)
    assert np.isfinite(out).all() and np.isfinite(lse).all()
    # short runs of consecutive rows (one oracle call each) on three of the eight KV heads with their query heads
    runs = [(0, 2), (31, 34), (255, 258), (2047, 2049), (3333, 3334), (3838, 3841), (4093, 4096)]
    heads = [0, 3, 7]
    g = h_q // h_kv
    q_heads = [h * g + i for h in heads for i in range(g)]
    kc64, vc64, kb64, vb64 = f64(kc[heads]), f64(vc[heads]), f64(kb[heads]), f64(vb[heads])
    worst, worst_l, n_rows = 0.0, 0.0, 0
    for j0, j1 in runs:
        args = dict(block_pos0=block_pos0, q_pos0=block_pos0 + j0)
        qq = f64(q[q_heads, j0:j1])
        o_out, o_lse = O.attend_block(qq, kc64, vc64, n, kb64, vb64, **args)
        scale, _ = O.attend_block(qq, kc64, np.abs(vc64), n, kb64, np.abs(vb64), **args)
        err = np.abs(out[q_heads, j0:j1].astype(np.float64) - o_out)
        assert np.all(err <= TOL["bf16"] * (np.abs(o_out) + scale)), f"rows {j0}..{j1 - 1}: output beyond tolerance"
        worst = max(worst, float((err / (np.abs(o_out) + scale)).max()))
        worst_l = max(worst_l, float(np.abs(lse[q_heads, j0:j1].astype(np.float64) - o_lse).max()))
        n_rows += j1 - j0
    assert worst <= OBSERVED["bf16"] and worst_l <= 1e-4
    say(f"[attend_block 128k last block] {n_rows} sampled rows x {len(q_heads)} query heads: max err/(|o|+scale) {worst:.2e}, max |lse diff| {worst_l:.2e}")
    lib.close()


def test_block_loop_with_attention_under_graph_replay():
    """The whole block loop of a layer (attention, window statistics, one sweep, select + append per block)
    captured once and replayed three times with eager launches and synchronisations of its own in between:
    every replay must leave the cache, the positions, the last block's attention output and its log-sum-exp
    exactly as the eager run left them."""
    from paper_2602_02199_amd.driver import LayerCompressor
    wl = synth.shrink(synth.WORKLOADS["llama8b-16k"], index=41, l_ctx=8192)
    comp = LayerCompressor(wl, DEV)
    data = synth.make_layer(wl, 1, comp.parts[0])
    ddev = {k: v.to(DEV) for k, v in data.items() if k != "needles"}
    s, d, w, nb = wl.s_block, wl.head_dim, wl.window, wl.n_blocks
    gen = torch.Generator().manual_seed(9)
    q_blocks = []
    for t in range(nb):
        q = torch.randn(wl.n_q_heads, s, d, generator=gen).to(wl.torch_dtype)
        q[:, s - w:] = data["q_win"][t]
        q_blocks.append(q.to(DEV))
    out = torch.empty(wl.n_q_heads, s, d, dtype=torch.float32, device=DEV)
    lse = torch.empty(wl.n_q_heads, s, dtype=torch.float32, device=DEV)
    lse_win = torch.empty(wl.n_q_heads, w, dtype=torch.float32, device=DEV)
    n_last = (nb - 1) * comp.B
    ws = torch.empty(max(comp.lib.laserkv_attend_block_workspace_bytes(s, n, s) for n in (0, n_last)), dtype=torch.uint8, device=DEV)
    run = lambda: comp.run_layer_with_attention(ddev, q_blocks, out, lse, lse_win, ws)

    def state():
        torch.cuda.synchronize()
        return [t.cpu().clone() for t in (comp.k_cache, comp.v_cache, comp.cache_pos, out, lse, lse_win)]

    def scrub():
        for t in (comp.k_cache, comp.v_cache, out, lse, lse_win):
            t.fill_(float("nan"))
        comp.cache_pos.fill_(-7)

    assert run() == nb * comp.B
    want = state()
    assert torch.isfinite(want[3]).all() and (want[2] >= 0).all()
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(stream):
        run()
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            run()
    for rnd in range(3):
        scrub()                      # eager work between the replays
        torch.cuda.synchronize()
        graph.replay()
        got = state()
        for name, a, b in zip(("k_cache", "v_cache", "cache_pos", "out", "lse", "lse_win"), want, got):
            assert torch.equal(a, b), f"replay {rnd}: {name} differs from the eager run"
    say(f"[attend_block graph] {nb} blocks captured, 3 replays identical to the eager run")
    comp.lib.close()
