"""GPU tests of the one-sweep path taken when the caller supplies complete row statistics
(laserkv_set_row_lse_complete; Sec. 3.3 "Precision"): parity with the oracle, agreement with the two-sweep
path, the bounded wait on other workgroups' histograms (forced from the host to expire at once), and
replays of a captured launch on changing inputs."""
import numpy as np
import pytest
import torch

from oracle import laserkv_oracle as O
from paper_2602_02199_amd import binding, synth
from tests.parity_util import check_block
from tests.test_gpu_parity import DEV, complete_row_lse, dbg_buffers, f64, gpu_stage, say, to_dev

pytestmark = pytest.mark.gpu


def run_blocks(wl, data, dev, parts, nb, lses):
    """select_block in complete-LSE mode for the first nb blocks; returns per-block stage outputs and how many
    launches of each kernel kind the context made."""
    na, nl, ke, kl = parts
    s, d = wl.s_block, wl.head_dim
    lib = binding.LaserKV(wl.n_q_heads, wl.n_kv_heads, d, wl.dtype, wl.lsh_tables, wl.lsh_bits,
                          max_block=s, max_window=wl.window, max_ctx_keys=0)
    lib.laserkv_profile_begin()
    outs = []
    for t in range(nb):
        lo = t * s
        lse_dev = lses[t].to(DEV)
        lib.laserkv_set_row_lse_complete(lse_dev)
        dbg = dbg_buffers(wl, s)
        keep = torch.empty(wl.n_kv_heads, sum(parts), dtype=torch.int32, device=DEV)
        lib.laserkv_select_block(dev["q_win"][t], dev["k"][:, lo:lo + s], None, dev["planes"], block_pos0=lo,
                                 n_anchor=na, n_local=nl, k_exact=ke, k_lsh=kl, keep_idx=keep,
                                 dbg_s_exact=dbg["s_exact"], dbg_sig_k=dbg["sig_k"], dbg_sig_q=dbg["sig_q"], dbg_count=dbg["cnt"])
        torch.cuda.synchronize()
        outs.append(gpu_stage(dbg, keep))
    launches = {k: v[1] for k, v in lib.laserkv_profile_end().items()}
    lib.laserkv_set_row_lse_complete(None)
    lib.close()
    return outs, launches


@pytest.mark.parametrize("name,kw,nb", [("tiny", dict(l_ctx=2048), 4), ("llama8b-16k", dict(l_ctx=4096), 2),
                                        ("llama8b-128k", dict(l_ctx=16384), 3), ("llama8b-128k", dict(l_ctx=12288, s_block=1000), 2)])
def test_single_sweep_against_oracle_and_both_other_routes(name, kw, nb, monkeypatch):
    wl = synth.shrink(synth.WORKLOADS[name], index=23, **kw)
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    parts = O.partition(B, wl.n_div, wl.alpha, wl.s_block)
    nl = parts[1]
    data = synth.make_layer(wl, 2, parts[0], n_blocks=nb)
    dev = to_dev(data)
    s, d = wl.s_block, wl.head_dim
    lses = []
    for t in range(nb):
        lo = t * s
        lses.append(complete_row_lse(data["q_win"][t], data["k"][:, lo:lo + s], data["k"][:, lo - nl:lo] if t else None,
                                     s - wl.window, d))
    res = {}
    for tag, spin in (("single", None), ("no-wait", "0"), ("two-sweeps", "-1")):
        if spin is None:
            monkeypatch.delenv("LASERKV_SINGLE_SPIN", raising=False)
        else:
            monkeypatch.setenv("LASERKV_SINGLE_SPIN", spin)
        say(f"[single {wl.name} s_t {s}] route {tag}")
        res[tag] = run_blocks(wl, data, dev, parts, nb, lses)
    assert res["single"][1]["single"] == nb and res["single"][1]["sweep1"] == 0
    assert res["no-wait"][1]["single"] == nb
    assert res["two-sweeps"][1]["single"] == 0 and res["two-sweeps"][1]["sweep1"] == nb
    for t in range(nb):
        lo = t * s
        st = O.select_block(f64(data["q_win"][t]), f64(data["k"][:, lo:lo + s]), None, f64(data["planes"]), wl.lsh_tables,
                            wl.lsh_bits, *parts, block_pos0=lo, row_lse_complete=lses[t].to(torch.float64).numpy())
        a, b, c = res["single"][0][t], res["no-wait"][0][t], res["two-sweeps"][0][t]
        rep = check_block(st, a, parts, wl.dtype)
        say(f"[single {wl.name} blk {t}] max score err/(s+s_k) {rep['max_rel']:.2e}, tolerated {rep['tolerated']}")
        # a workgroup that computes a table itself writes the same histogram: bit-identical results
        for key in ("s_exact", "sig_k", "sig_q", "cnt", "keep"):
            assert np.array_equal(a[key], b[key]), f"block {t}: {key} differs when no flag is waited for"
        # the two-sweep route hashes and counts identically and sums the same probabilities in another order
        for key in ("sig_k", "sig_q", "cnt"):
            assert np.array_equal(a[key], c[key]), f"block {t}: {key} differs from the two-sweep route"
        x, y = a["s_exact"].astype(np.float64), c["s_exact"].astype(np.float64)
        assert np.all(np.abs(x - y) <= 1e-5 * np.maximum(x, y) + 1e-30)


def test_single_sweep_graph_replays_on_changing_inputs():
    """One captured laserkv_compress_block (complete statistics) replayed on three different blocks copied into
    the same buffers: every replay must equal the eager result for that block.  The flags of an earlier launch
    must never pass for those of the running one."""
    wl = synth.shrink(synth.WORKLOADS["llama8b-128k"], index=29, l_ctx=16384)
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    parts = O.partition(B, wl.n_div, wl.alpha, wl.s_block)
    na, nl, ke, kl = parts
    nb = 3
    data = synth.make_layer(wl, 3, na, n_blocks=nb)
    dev = to_dev(data)
    s, d, w = wl.s_block, wl.head_dim, wl.window
    lses = [complete_row_lse(data["q_win"][t], data["k"][:, t * s:(t + 1) * s], None, s - w, d).to(DEV) for t in range(nb)]
    lib = binding.LaserKV(wl.n_q_heads, wl.n_kv_heads, d, wl.dtype, wl.lsh_tables, wl.lsh_bits,
                          max_block=s, max_window=w, max_ctx_keys=0)
    cap = nb * B
    q_buf, k_buf, v_buf = torch.empty_like(dev["q_win"][0]), torch.empty_like(dev["k"][:, :s]), torch.empty_like(dev["v"][:, :s])
    lse_buf = torch.empty_like(lses[0])
    keep = torch.empty(wl.n_kv_heads, B, dtype=torch.int32, device=DEV)

    def fresh_cache():
        return (torch.zeros(wl.n_kv_heads, cap, d, dtype=wl.torch_dtype, device=DEV),
                torch.zeros(wl.n_kv_heads, cap, d, dtype=wl.torch_dtype, device=DEV),
                torch.full((wl.n_kv_heads, cap), -1, dtype=torch.int64, device=DEV))

    def load(t):
        q_buf.copy_(dev["q_win"][t]); k_buf.copy_(dev["k"][:, t * s:(t + 1) * s]); v_buf.copy_(dev["v"][:, t * s:(t + 1) * s])
        lse_buf.copy_(lses[t])

    lib.laserkv_set_row_lse_complete(lse_buf)
    kc, vc, pc = fresh_cache()

    def call(stream=None):
        lib.laserkv_compress_block(q_buf, k_buf, v_buf, None, dev["planes"], block_pos0=0, n_anchor=na, n_local=nl,
                                   k_exact=ke, k_lsh=kl, keep_idx=keep, k_cache=kc, v_cache=vc, cache_pos=pc, cache_len=0,
                                   stream=stream)

    eager = []
    for t in range(nb):
        load(t)
        call()
        torch.cuda.synchronize()
        eager.append((keep.cpu().numpy().copy(), kc[:, :B].cpu().clone()))
    assert not np.array_equal(eager[0][0], eager[1][0])
    stream = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    load(0)
    torch.cuda.synchronize()
    with torch.cuda.stream(stream):
        call(stream.cuda_stream)   # warm-up on the capture stream
        stream.synchronize()
        with torch.cuda.graph(graph, stream=stream):
            call(stream.cuda_stream)
    for rnd in range(2):
        for t in (2, 0, 1):
            load(t)
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            assert np.array_equal(keep.cpu().numpy(), eager[t][0]), f"replay round {rnd} block {t}: kept set differs"
            assert torch.equal(kc[:, :B].cpu(), eager[t][1]), f"replay round {rnd} block {t}: cache rows differ"
    lib.laserkv_set_row_lse_complete(None)
    lib.close()


def test_single_sweep_counts_equal_the_two_sweep_route_over_many_launches(monkeypatch):
    """The collision counts of the one-sweep route depend on histograms that other workgroups publish during the
    same launch.  Sixteen blocks of four layers, each launched five times in a row through one context, must give
    the counts, codes and kept sets of the two-sweep route (whose histograms cross a kernel boundary) every time."""
    wl = synth.shrink(synth.WORKLOADS["llama8b-128k"], index=31, l_ctx=16384)
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    parts = O.partition(B, wl.n_div, wl.alpha, wl.s_block)
    na, nl, ke, kl = parts
    s, d, w = wl.s_block, wl.head_dim, wl.window
    monkeypatch.setenv("LASERKV_SINGLE_SPIN", "-1")
    two = binding.LaserKV(wl.n_q_heads, wl.n_kv_heads, d, wl.dtype, wl.lsh_tables, wl.lsh_bits, max_block=s, max_window=w,
                          max_ctx_keys=0)
    monkeypatch.delenv("LASERKV_SINGLE_SPIN")
    one = binding.LaserKV(wl.n_q_heads, wl.n_kv_heads, d, wl.dtype, wl.lsh_tables, wl.lsh_bits, max_block=s, max_window=w,
                          max_ctx_keys=0)
    n_checked = 0
    for layer in range(4):
        data = synth.make_layer(wl, layer, na, n_blocks=4)
        dev = to_dev(data)
        for t in range(4):
            lo = t * s
            lse = complete_row_lse(data["q_win"][t], data["k"][:, lo:lo + s], None, s - w, d).to(DEV)
            res = []
            for lib, reps in ((two, 1), (one, 5)):
                lib.laserkv_set_row_lse_complete(lse)
                for _ in range(reps):
                    dbg = dbg_buffers(wl, s)
                    keep = torch.empty(wl.n_kv_heads, sum(parts), dtype=torch.int32, device=DEV)
                    lib.laserkv_select_block(dev["q_win"][t], dev["k"][:, lo:lo + s], None, dev["planes"], block_pos0=lo,
                                             n_anchor=na, n_local=nl, k_exact=ke, k_lsh=kl, keep_idx=keep,
                                             dbg_s_exact=dbg["s_exact"], dbg_sig_k=dbg["sig_k"], dbg_sig_q=dbg["sig_q"],
                                             dbg_count=dbg["cnt"])
                    res.append(gpu_stage(dbg, keep))
            torch.cuda.synchronize()
            ref = res[0]
            for i, r in enumerate(res[1:]):
                for key in ("cnt", "sig_k", "sig_q"):
                    assert np.array_equal(ref[key], r[key]), f"layer {layer} block {t} launch {i}: {key} differs"
                assert np.array_equal(res[1]["keep"], r["keep"]) and np.array_equal(res[1]["s_exact"], r["s_exact"])
                n_checked += 1
    say(f"[single] {n_checked} launches checked against the two-sweep route")
    for lib in (one, two):
        lib.laserkv_set_row_lse_complete(None)
        lib.close()
