"""GPU parity: the HIP path through the C-ABI against the CPU oracle on the same seeded inputs."""
import sys

import numpy as np
import pytest
import torch

from oracle import laserkv_oracle as O
from paper_2602_02199_amd import binding, synth
from paper_2602_02199_amd.driver import LayerCompressor
from tests.parity_util import check_block

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def say(msg):
    print(msg, flush=True)
    sys.stdout.flush()


def to_dev(data):
    return {k: (v.to(DEV) if k != "needles" else v) for k, v in data.items()}


def f64(t):
    return t.detach().cpu().to(torch.float64).numpy()


def dbg_buffers(wl, s_t):
    return dict(
        s_exact=torch.empty(wl.n_kv_heads, s_t, dtype=torch.float32, device=DEV),
        sig_k=torch.empty(wl.n_kv_heads, s_t, wl.lsh_tables, dtype=torch.int16, device=DEV),
        sig_q=torch.empty(wl.n_q_heads, wl.window, wl.lsh_tables, dtype=torch.int16, device=DEV),
        cnt=torch.empty(wl.n_kv_heads, s_t, dtype=torch.int32, device=DEV),
    )


def gpu_stage(dbg, keep):
    return dict(
        s_exact=dbg["s_exact"].cpu().numpy(),
        sig_k=dbg["sig_k"].cpu().numpy().view(np.uint16),
        sig_q=dbg["sig_q"].cpu().numpy().view(np.uint16),
        cnt=dbg["cnt"].cpu().numpy(),
        keep=keep.cpu().numpy(),
    )


def run_and_check(wl, layer=0, n_blocks=None, check_blocks=None, label="", mutate=None):
    """Run the layer's blocks on the GPU in the benchmark's launch configuration; check the listed
    blocks stage by stage against the oracle, and whole-run invariants on the cache.
    mutate(data) may alter the generated inputs in place (both sides then see the altered values)."""
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    parts_full = O.partition(B, wl.n_div, wl.alpha, wl.s_block)
    data = synth.make_layer(wl, layer, parts_full[0], n_blocks=n_blocks)
    if mutate is not None:
        mutate(data)
    nb = data["q_win"].shape[0]
    check_blocks = list(range(nb)) if check_blocks is None else check_blocks
    dev = to_dev(data)
    comp = LayerCompressor(wl, DEV)
    assert comp.B == B and comp.parts == parts_full
    l_tot = data["k"].shape[1]
    prev_local, saved = 0, {}
    for t in range(nb):
        lo, hi = t * wl.s_block, min((t + 1) * wl.s_block, l_tot)
        dbg = dbg_buffers(wl, hi - lo) if t in check_blocks else None
        keep_out = None
        if t in check_blocks:
            b_t = sum(O.partition(B, wl.n_div, wl.alpha, hi - lo))
            keep_out = torch.empty(wl.n_kv_heads, b_t, dtype=torch.int32, device=DEV)
        n_ctx = prev_local
        prev_local, keep = comp.step(dev["q_win"][t], dev["k"][:, lo:hi], dev["v"][:, lo:hi], dev["planes"], lo,
                                     prev_local, dbg=dbg, keep_out=keep_out)
        if t in check_blocks:
            saved[t] = (dbg, keep, n_ctx)
    torch.cuda.synchronize()
    k64, planes64 = f64(data["k"]), f64(data["planes"])
    reports = []
    for t in check_blocks:
        dbg, keep, n_ctx = saved[t]
        lo, hi = t * wl.s_block, min((t + 1) * wl.s_block, l_tot)
        parts = O.partition(B, wl.n_div, wl.alpha, hi - lo)
        k_ctx = k64[:, lo - n_ctx:lo] if n_ctx else None      # previous block's local window
        st = O.select_block(f64(data["q_win"][t]), k64[:, lo:hi], k_ctx, planes64, wl.lsh_tables, wl.lsh_bits,
                            *parts, block_pos0=lo)
        rep = check_block(st, gpu_stage(dbg, keep), parts, wl.dtype)
        reports.append(rep)
        say(f"[{label or wl.name} L{layer} blk {t}] unsure codes k/q {rep['unsure_k']}/{rep['unsure_q']}, "
            f"max score err/(s+s_k) {rep['max_rel']:.2e}, tolerated index diffs per head {rep['tolerated']}")
    # whole-run invariants on the device cache
    n = comp.cache_len
    pos = comp.cache_pos[:, :n]
    assert n == sum(sum(O.partition(B, wl.n_div, wl.alpha, min(wl.s_block, l_tot - t * wl.s_block))) for t in range(nb))
    assert bool((pos[:, 1:] > pos[:, :-1]).all()), "cache positions not strictly increasing"
    assert bool((comp.cache_pos[:, n:] == -1).all()), "rows past the cache length were written"
    gk = torch.gather(dev["k"], 1, pos[:, :, None].expand(-1, -1, wl.head_dim))
    gv = torch.gather(dev["v"], 1, pos[:, :, None].expand(-1, -1, wl.head_dim))
    assert torch.equal(gk, comp.k_cache[:, :n]) and torch.equal(gv, comp.v_cache[:, :n]), "cache rows are not verbatim copies"
    off = 0
    for t in range(nb):
        lo = t * wl.s_block
        b_t = sum(O.partition(B, wl.n_div, wl.alpha, min(wl.s_block, l_tot - lo)))
        if t in saved:
            assert torch.equal(pos[:, off:off + b_t], saved[t][1].to(torch.int64) + lo)
        off += b_t
    return data, comp, reports


def test_tiny_fp32_all_blocks():
    wl = synth.WORKLOADS["tiny"]
    data, comp, reps = run_and_check(wl)
    kept = {(int(p) // wl.s_block, h, int(p) % wl.s_block) for h in range(wl.n_kv_heads)
            for p in comp.cache_pos[h, :comp.cache_len].cpu().tolist()}
    for blk, h, p in data["needles"].tolist():
        assert (blk, h, p) in kept


def test_llama16k_bf16_all_blocks():
    run_and_check(synth.WORKLOADS["llama8b-16k"])


@pytest.mark.parametrize("case", [
    dict(name="ragged-bf16-d64", n_q_heads=6, n_kv_heads=2, head_dim=64, dtype="bf16", l_ctx=2500, s_block=1000,
         window=24, n_div=5, lsh_tables=5, lsh_bits=7),
    dict(name="ragged-f32-d128", n_q_heads=3, n_kv_heads=3, head_dim=128, dtype="f32", l_ctx=700, s_block=333,
         window=17, n_div=3, lsh_tables=3, lsh_bits=11),
    dict(name="wide-rows-bf16", n_q_heads=16, n_kv_heads=1, head_dim=128, dtype="bf16", l_ctx=1536, s_block=768,
         window=40, n_div=4, lsh_tables=31, lsh_bits=16),
    dict(name="one-table-one-bit", n_q_heads=2, n_kv_heads=2, head_dim=64, dtype="f32", l_ctx=130, s_block=65,
         window=3, n_div=2, lsh_tables=1, lsh_bits=1),
    # the longest block a context accepts (16384 keys: 16 positions per select thread)
    dict(name="max-block", n_q_heads=1, n_kv_heads=1, head_dim=64, dtype="bf16", l_ctx=16384, s_block=16384,
         window=8, n_div=8, lsh_tables=2, lsh_bits=5),
    # the most window rows a head may have (G*W = 1024: four query-row groups)
    dict(name="max-rows", n_q_heads=16, n_kv_heads=1, head_dim=64, dtype="f32", l_ctx=640, s_block=320,
         window=64, n_div=4, lsh_tables=2, lsh_bits=6),
    # protection divisor larger than the budget: no anchors, no local window, no look-back keys
    dict(name="no-protected", n_q_heads=2, n_kv_heads=1, head_dim=64, dtype="f32", l_ctx=128, s_block=64,
         window=4, n_div=32, lsh_tables=2, lsh_bits=3),
    # one window query, one head, blocks shorter than a tile
    dict(name="one-query", n_q_heads=1, n_kv_heads=1, head_dim=128, dtype="bf16", l_ctx=57, s_block=19,
         window=1, n_div=2, lsh_tables=2, lsh_bits=2),
    # bit-wise scoring: 64 tables of one sign bit each (count = rows*tables - summed Hamming distance)
    dict(name="bitwise-64x1", n_q_heads=4, n_kv_heads=2, head_dim=64, dtype="bf16", l_ctx=900, s_block=450,
         window=16, n_div=4, lsh_tables=64, lsh_bits=1),
    # 768 window rows = three query-row groups, with the histogram path (K <= 12)
    dict(name="three-row-groups", n_q_heads=12, n_kv_heads=1, head_dim=128, dtype="bf16", l_ctx=1800, s_block=900,
         window=64, n_div=4, lsh_tables=6, lsh_bits=9),
    # 512 window rows x 4 tables of 2 bits: collision counts in the hundreds (two radix digits in stage 2)
    dict(name="big-counts", n_q_heads=8, n_kv_heads=1, head_dim=64, dtype="bf16", l_ctx=1200, s_block=600,
         window=64, n_div=4, lsh_tables=4, lsh_bits=2),
    # more query-row groups than tables: the groups without a table contribute no count part
    dict(name="two-row-groups-one-table", n_q_heads=5, n_kv_heads=1, head_dim=64, dtype="bf16", l_ctx=1000, s_block=500,
         window=64, n_div=4, lsh_tables=1, lsh_bits=5),
    dict(name="four-row-groups-three-tables", n_q_heads=16, n_kv_heads=1, head_dim=128, dtype="bf16", l_ctx=800,
         s_block=400, window=64, n_div=4, lsh_tables=3, lsh_bits=4),
    # the widest rows with the longest block a context accepts: the finest key-range split
    dict(name="max-block-f32-d128", n_q_heads=2, n_kv_heads=1, head_dim=128, dtype="f32", l_ctx=16384, s_block=16384,
         window=8, n_div=8, lsh_tables=4, lsh_bits=8),
])
def test_ragged_shapes(case):
    base = synth.WORKLOADS["tiny"]
    wl = synth.shrink(base, index=7, needles_per_block=2, outlier_channels=2, **case)
    run_and_check(wl, label=case["name"])


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_dominant_late_key(dtype):
    """Keys deep inside a key range whose logit for one window row lies ~120 nats above everything the
    row has seen before: the first sweep's running sums overflow against the first tile's maximum and
    the kernel has to redo those rows with a reference that follows the maximum."""
    wl = synth.shrink(synth.WORKLOADS["llama8b-16k"], index=9, l_ctx=4096, dtype=dtype, needles_per_block=2)
    d, g = wl.head_dim, wl.group
    planted = []

    def mutate(data):
        k = data["k"].to(torch.float32)
        for t in range(data["q_win"].shape[0]):
            for h in range(wl.n_kv_heads):
                for i, (gi, j) in ((360 + 7 * h, (h % g, 5)), (1201 + 3 * h, ((h + 1) % g, wl.window - 1))):
                    qv = data["q_win"][t, h * g + gi, j].to(torch.float32)
                    k[h, t * wl.s_block + i] = qv * (120.0 * d ** 0.5 / float(qv @ qv))
                    planted.append((t, h, i))
        data["k"] = k.to(wl.torch_dtype).contiguous()

    _, comp, reps = run_and_check(wl, label=f"dominant-late-key-{dtype}", mutate=mutate)
    kept = {(int(p) // wl.s_block, h, int(p) % wl.s_block) for h in range(wl.n_kv_heads)
            for p in comp.cache_pos[h, :comp.cache_len].cpu().tolist()}
    assert all(x in kept for x in planted)


@pytest.mark.parametrize("alpha", [0.0, 1.0, 0.5])
def test_alpha_end_points(alpha):
    wl = synth.shrink(synth.WORKLOADS["tiny"], alpha=alpha, l_ctx=1024)
    run_and_check(wl, label=f"tiny-alpha{alpha}")


def test_llama128k_full_size_every_block():
    wl = synth.WORKLOADS["llama8b-128k"]
    run_and_check(wl)


def test_gqa8_128k_full_size_sampled_blocks():
    wl = synth.WORKLOADS["gqa8-128k"]
    run_and_check(wl, check_blocks=[0, 15])


def test_llama64k_four_layers_sampled_blocks():
    wl = synth.WORKLOADS["llama8b-64k"]
    for layer in (0, 10, 21, 31):
        run_and_check(wl, layer=layer, check_blocks=[0, 16, 31])


def test_count_parts_on_a_poisoned_workspace(monkeypatch):
    """LASERKV_POISON_WORKSPACE=1 (read when a context is created) fills the fresh workspace with a non-zero
    pattern.  With more query-row groups than tables some groups write no count part; the selection must
    not read those parts, whatever the workspace held before."""
    monkeypatch.setenv("LASERKV_POISON_WORKSPACE", "1")
    base = synth.WORKLOADS["tiny"]
    for case in (dict(name="poison-2-groups-1-table", n_q_heads=5, n_kv_heads=1, head_dim=64, dtype="bf16", l_ctx=1000,
                      s_block=500, window=64, n_div=4, lsh_tables=1, lsh_bits=5),
                 dict(name="poison-4-groups-2-tables", n_q_heads=16, n_kv_heads=1, head_dim=64, dtype="f32", l_ctx=640,
                      s_block=320, window=64, n_div=4, lsh_tables=2, lsh_bits=6),
                 dict(name="poison-4-groups-3-tables", n_q_heads=16, n_kv_heads=2, head_dim=128, dtype="bf16", l_ctx=800,
                      s_block=400, window=64, n_div=4, lsh_tables=3, lsh_bits=4)):
        wl = synth.shrink(base, index=23, needles_per_block=2, outlier_channels=2, **case)
        run_and_check(wl, label=case["name"])


def test_repeat_runs_are_bit_identical():
    wl = synth.WORKLOADS["llama8b-16k"]
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    na = O.partition(B, wl.n_div, wl.alpha, wl.s_block)[0]
    dev = to_dev(synth.make_layer(wl, 3, na, n_blocks=2))
    comp = LayerCompressor(wl, DEV, max_blocks=2)
    ref = None
    for _ in range(5):
        comp.run_layer(dev)
        torch.cuda.synchronize()
        cur = (comp.cache_pos.clone(), comp.k_cache.clone())
        if ref is None:
            ref = cur
        assert torch.equal(ref[0], cur[0]) and torch.equal(ref[1], cur[1])


def test_error_paths_return_codes_and_launch_nothing():
    wl = synth.WORKLOADS["tiny"]
    lib = binding.LaserKV(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.dtype, wl.lsh_tables, wl.lsh_bits,
                          max_block=512, max_window=32, max_ctx_keys=56)
    q = torch.zeros(4, 32, 64, device=DEV)
    k = torch.zeros(2, 512, 64, device=DEV)
    planes = torch.zeros(64, 64, device=DEV)
    keep = torch.full((2, 227), -7, dtype=torch.int32, device=DEV)
    ok = dict(block_pos0=0, n_anchor=56, n_local=56, k_exact=86, k_lsh=29, keep_idx=keep)
    bad_calls = [
        dict(ok, k_exact=500),                                   # recall budget > candidates
        dict(ok, n_anchor=400, n_local=400),                     # protected sets exceed the block
        dict(ok, q_pos0=-5),                                     # causal window before the block
    ]
    for kw in bad_calls:
        with pytest.raises(binding.LaserKVError) as ei:
            lib.laserkv_select_block(q, k, None, planes, **kw)
        assert ei.value.code == binding.LKV_EINVAL
    with pytest.raises(binding.LaserKVError):                    # block longer than the configured maximum
        lib.laserkv_select_block(q, torch.zeros(2, 600, 64, device=DEV), None, planes, **ok)
    with pytest.raises(binding.LaserKVError):                    # look-back keys beyond the configured maximum
        lib.laserkv_select_block(q, k, torch.zeros(2, 100, 64, device=DEV), planes, **ok)
    torch.cuda.synchronize()
    assert bool((keep == -7).all())
    kc = torch.zeros(2, 300, 64, device=DEV)
    pos = torch.zeros(2, 300, dtype=torch.int64, device=DEV)
    with pytest.raises(binding.LaserKVError) as ei:
        lib.laserkv_append(k, k, keep, b_t=227, block_pos0=0, k_cache=kc, v_cache=kc.clone(), cache_pos=pos, cache_len=100)
    assert ei.value.code == binding.LKV_ECAP
    lib.close()


def test_graph_replay_matches_eager_every_time():
    """A captured layer (what bench.py times) must reproduce the eager result on every replay, with eager
    work and synchronisations between replays."""
    wl = synth.WORKLOADS["llama8b-16k"]
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    na = O.partition(B, wl.n_div, wl.alpha, wl.s_block)[0]
    dev = to_dev(synth.make_layer(wl, 5, na, n_blocks=3))
    comp = LayerCompressor(wl, DEV, max_blocks=3)
    plan = comp.plan_layer(dev)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        comp.run_plan(plan)
        stream.synchronize()
        ref = (comp.cache_pos.clone(), comp.k_cache.clone(), comp.v_cache.clone())
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            comp.run_plan(plan)
        for it in range(4):
            comp.cache_pos.fill_(-1)
            comp.k_cache.zero_()
            comp.v_cache.zero_()
            stream.synchronize()
            graph.replay()
            stream.synchronize()
            assert torch.equal(comp.cache_pos, ref[0]) and torch.equal(comp.k_cache, ref[1]) and torch.equal(comp.v_cache, ref[2]), it
            comp.run_plan(plan)          # eager work between replays
            stream.synchronize()
            assert torch.equal(comp.cache_pos, ref[0])


@pytest.mark.parametrize("name,n_blocks", [("tiny", 3), ("llama8b-16k", 2), ("gqa8-128k", 1)])
def test_compress_block_equals_select_then_append(name, n_blocks):
    """The one-call entry point must leave exactly the cache the two separate calls leave."""
    wl = synth.WORKLOADS[name]
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    na = O.partition(B, wl.n_div, wl.alpha, wl.s_block)[0]
    dev = to_dev(synth.make_layer(wl, 2, na, n_blocks=n_blocks))
    results = []
    for fused in (False, True):
        comp = LayerCompressor(wl, DEV, max_blocks=n_blocks)
        plan = comp.plan_layer(dev, fused=fused)
        comp.run_plan(plan)
        torch.cuda.synchronize()
        results.append((comp.cache_pos.clone(), comp.k_cache.clone(), comp.v_cache.clone(), comp.keep.clone()))
        assert comp.cache_len == n_blocks * min(B, wl.s_block)
    for a, b in zip(*results):
        assert torch.equal(a, b)
    assert bool((results[1][0][:, :n_blocks * min(B, wl.s_block)] >= 0).all())


def test_profile_isolate_restores_normal_operation():
    """laserkv_profile_isolate launches one kernel kind only (benchmarks); after it is switched off the
    same calls must again give the results of a complete pass."""
    wl = synth.WORKLOADS["llama8b-16k"]
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    na = O.partition(B, wl.n_div, wl.alpha, wl.s_block)[0]
    dev = to_dev(synth.make_layer(wl, 3, na, n_blocks=2))
    comp = LayerCompressor(wl, DEV, max_blocks=2)
    plan = comp.plan_layer(dev, fused=True)
    comp.run_plan(plan)
    torch.cuda.synchronize()
    want = (comp.cache_pos.clone(), comp.k_cache.clone(), comp.v_cache.clone())
    for name in ("sweep1", "sweep2", "select"):
        comp.lib.laserkv_profile_isolate(name)
        comp.run_plan(plan)
    comp.lib.laserkv_profile_isolate(None)
    with pytest.raises(binding.LaserKVError):
        comp.lib._check(comp.lib._lib.laserkv_profile_isolate(comp.lib._ctx, 99))
    comp.cache_pos.fill_(-1)
    comp.k_cache.zero_()
    comp.v_cache.zero_()
    comp.run_plan(plan)
    torch.cuda.synchronize()
    for a, b in zip(want, (comp.cache_pos, comp.k_cache, comp.v_cache)):
        assert torch.equal(a, b)


def test_separate_count_kernel_path(monkeypatch):
    """LASERKV_NO_QHIST=1 (read when a context is created) forces the stand-alone count kernel, which is
    otherwise used only when neither histograms nor code tables fit a call."""
    monkeypatch.setenv("LASERKV_NO_QHIST", "1")
    wl = synth.shrink(synth.WORKLOADS["llama8b-16k"], index=11, l_ctx=4096)
    run_and_check(wl, label="count-kernel-16x10")
    wl = synth.shrink(synth.WORKLOADS["tiny"], index=12, l_ctx=1024, lsh_tables=3, lsh_bits=16)
    run_and_check(wl, label="count-kernel-3x16")


@pytest.mark.parametrize("name,kw", [("tiny", dict(l_ctx=1024)), ("llama8b-16k", dict(l_ctx=2048))])
def test_row_lse_of_outside_keys(name, kw):
    """laserkv_set_row_lse: keys outside the call, summarised as one log-sum-exp per window query, join the
    normaliser; switching it off again restores the plain result."""
    wl = synth.shrink(synth.WORKLOADS[name], index=13, **kw)
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    parts = O.partition(B, wl.n_div, wl.alpha, wl.s_block)
    data = synth.make_layer(wl, 0, parts[0], n_blocks=1)
    dev = to_dev(data)
    s, d, g = wl.s_block, wl.head_dim, wl.group
    gen = torch.Generator().manual_seed(5)
    k_out = torch.randn(wl.n_kv_heads, 300, d, generator=gen, dtype=torch.float64) * 3.0
    q64 = data["q_win"][0].to(torch.float64)
    row_lse = torch.stack([torch.logsumexp(q64[hq] @ k_out[hq // g].T / d ** 0.5, dim=1) for hq in range(wl.n_q_heads)])
    row_lse = row_lse.to(torch.float32).contiguous()            # both sides use these rounded values
    lib = binding.LaserKV(wl.n_q_heads, wl.n_kv_heads, d, wl.dtype, wl.lsh_tables, wl.lsh_bits,
                          max_block=s, max_window=wl.window, max_ctx_keys=0)
    outs = {}
    for tag, lse in (("with", row_lse.to(DEV)), ("without", None)):
        lib.laserkv_set_row_lse(lse)
        dbg = dbg_buffers(wl, s)
        keep = torch.empty(wl.n_kv_heads, sum(parts), dtype=torch.int32, device=DEV)
        lib.laserkv_select_block(dev["q_win"][0], dev["k"][:, :s], None, dev["planes"], block_pos0=0,
                                 n_anchor=parts[0], n_local=parts[1], k_exact=parts[2], k_lsh=parts[3], keep_idx=keep,
                                 dbg_s_exact=dbg["s_exact"], dbg_sig_k=dbg["sig_k"], dbg_sig_q=dbg["sig_q"], dbg_count=dbg["cnt"])
        torch.cuda.synchronize()
        outs[tag] = gpu_stage(dbg, keep)
    for tag, lse in (("with", row_lse.to(torch.float64).numpy()), ("without", None)):
        st = O.select_block(f64(data["q_win"][0]), f64(data["k"][:, :s]), None, f64(data["planes"]), wl.lsh_tables,
                            wl.lsh_bits, *parts, block_pos0=0, row_lse=lse)
        rep = check_block(st, outs[tag], parts, wl.dtype)
        say(f"[row-lse {wl.name} {tag}] max score err/(s+s_k) {rep['max_rel']:.2e}, tolerated {rep['tolerated']}")
    # the outside keys take a share of the probability mass
    assert outs["with"]["s_exact"].sum() < 0.99 * outs["without"]["s_exact"].sum()


def complete_row_lse(q_win, k_blk, k_ctx, q_pos0_minus_block_pos0, d):
    """float32 [H_q, W]: log-sum-exp of every window row over the look-back keys and the block keys it sees
    (torch float64 on the CPU: stands in for what the model's attention kernel reports)."""
    h_q, w, _ = q_win.shape
    h_kv, s_t, _ = k_blk.shape
    g = h_q // h_kv
    vis = torch.arange(s_t)[None, :] <= (q_pos0_minus_block_pos0 + torch.arange(w))[:, None]
    out = torch.empty(h_q, w, dtype=torch.float64)
    for hq in range(h_q):
        h = hq // g
        l_blk = (q_win[hq].double() @ k_blk[h].double().T / d ** 0.5).masked_fill(~vis, float("-inf"))
        parts = [l_blk] if k_ctx is None else [q_win[hq].double() @ k_ctx[h].double().T / d ** 0.5, l_blk]
        out[hq] = torch.logsumexp(torch.cat(parts, dim=1), dim=1)
    return out.to(torch.float32).contiguous()


@pytest.mark.parametrize("name,kw", [("tiny", dict(l_ctx=1024)), ("llama8b-16k", dict(l_ctx=4096)),
                                     ("llama8b-128k", dict(l_ctx=8192)), ("gqa8-128k", dict(l_ctx=8192))])
def test_complete_row_lse_from_the_attention_kernel(name, kw):
    """laserkv_set_row_lse_complete: with every window row's complete log-sum-exp supplied (as the model's
    attention kernel reports it) the first sweep computes no row statistics and the look-back keys are not
    read; scores, codes, counts and kept sets must still match the oracle, and the scores must match what the
    library computes on its own from the same keys."""
    wl = synth.shrink(synth.WORKLOADS[name], index=17, **kw)
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    parts = O.partition(B, wl.n_div, wl.alpha, wl.s_block)
    na, nl, ke, kl = parts
    nb = min(2, wl.n_blocks)
    data = synth.make_layer(wl, 1, na, n_blocks=nb)
    dev = to_dev(data)
    s, d = wl.s_block, wl.head_dim
    lib = binding.LaserKV(wl.n_q_heads, wl.n_kv_heads, d, wl.dtype, wl.lsh_tables, wl.lsh_bits,
                          max_block=s, max_window=wl.window, max_ctx_keys=nl)
    for t in range(nb):
        lo = t * s
        k_blk = data["k"][:, lo:lo + s]
        k_ctx = data["k"][:, lo - nl:lo] if t else None
        lse = complete_row_lse(data["q_win"][t], k_blk, k_ctx, s - wl.window, d)
        outs = {}
        for tag in ("own", "complete"):
            lib.laserkv_set_row_lse_complete(lse.to(DEV) if tag == "complete" else None)
            dbg = dbg_buffers(wl, s)
            keep = torch.empty(wl.n_kv_heads, sum(parts), dtype=torch.int32, device=DEV)
            # the complete mode gets no look-back keys at all: they are inside the log-sum-exp
            ctx_dev = dev["k"][:, lo - nl:lo] if (t and tag == "own") else None
            lib.laserkv_select_block(dev["q_win"][t], dev["k"][:, lo:lo + s], ctx_dev, dev["planes"], block_pos0=lo,
                                     n_anchor=na, n_local=nl, k_exact=ke, k_lsh=kl, keep_idx=keep,
                                     dbg_s_exact=dbg["s_exact"], dbg_sig_k=dbg["sig_k"], dbg_sig_q=dbg["sig_q"], dbg_count=dbg["cnt"])
            torch.cuda.synchronize()
            outs[tag] = gpu_stage(dbg, keep)
        st = O.select_block(f64(data["q_win"][t]), f64(k_blk), None, f64(data["planes"]), wl.lsh_tables, wl.lsh_bits,
                            *parts, block_pos0=lo, row_lse_complete=lse.to(torch.float64).numpy())
        rep = check_block(st, outs["complete"], parts, wl.dtype)
        say(f"[complete-lse {wl.name} blk {t}] max score err/(s+s_k) {rep['max_rel']:.2e}, tolerated {rep['tolerated']}")
        # the library's own statistics over the same keys give the same scores up to the rounding of the
        # float32 log-sum-exp handed in (relative 2^-24 of a value around 10: a few 1e-6 in the exponent)
        own, comp = outs["own"]["s_exact"].astype(np.float64), outs["complete"]["s_exact"].astype(np.float64)
        assert np.all(np.abs(own - comp) <= 2e-5 * np.maximum(own, comp) + 1e-30)
        assert np.array_equal(outs["own"]["sig_k"], outs["complete"]["sig_k"]) and np.array_equal(outs["own"]["cnt"], outs["complete"]["cnt"])
    lib.laserkv_set_row_lse_complete(None)
    lib.close()


def test_bench_launch_configuration_full_size_against_oracle():
    """Exactly what bench.py times (the 128k layer as one captured graph of laserkv_compress_block calls,
    replayed): the rows in the cache for sampled blocks must be the oracle's kept rows, up to tokens at a
    selection threshold."""
    from tests.parity_util import TOL, count_interval
    wl = synth.WORKLOADS["llama8b-128k"]
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    parts = O.partition(B, wl.n_div, wl.alpha, wl.s_block)
    na, nl, ke, kl = parts
    data = synth.make_layer(wl, 0, na)
    dev = to_dev(data)
    comp = LayerCompressor(wl, DEV)
    plan = comp.plan_layer(dev, fused=True)
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        comp.run_plan(plan)
        stream.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            comp.run_plan(plan)
        comp.cache_pos.fill_(-1)
        comp.k_cache.zero_()
        stream.synchronize()
        graph.replay()
        graph.replay()
        stream.synchronize()
    s, b_t, tol = wl.s_block, sum(parts), TOL[wl.dtype]
    k64, planes64 = f64(data["k"]), f64(data["planes"])
    for t in (0, 17, 31):
        lo = t * s
        n_ctx = nl if t else 0
        st = O.select_block(f64(data["q_win"][t]), k64[:, lo:lo + s], k64[:, lo - n_ctx:lo] if n_ctx else None, planes64,
                            wl.lsh_tables, wl.lsh_bits, *parts, block_pos0=lo)
        got = (comp.cache_pos[:, t * b_t:(t + 1) * b_t] - lo).cpu().numpy()
        c_lo, c_hi = count_interval(st["sig_q"], st["sig_k"], st["unsure_q"], st["unsure_k"], wl.group)
        n_diff = 0
        for h in range(wl.n_kv_heads):
            assert np.all(np.diff(got[h]) > 0)
            diff = np.setxor1d(got[h], st["keep"][h])
            if diff.size:
                cand = np.arange(na, s - nl)
                s_k = np.sort(st["s_exact"][h][cand])[::-1][ke - 1]
                resid = np.setdiff1d(cand, st["k_exact_set"][h])
                c_k = np.sort(st["cnt"][h][resid])[::-1][kl - 1]
                for i in diff:
                    assert abs(st["s_exact"][h][i] - s_k) <= tol * s_k or c_lo[h, i] <= c_k <= c_hi[h, i], (t, h, int(i))
                n_diff += diff.size
        say(f"[bench configuration blk {t}] kept rows differing from the oracle's at a threshold: {n_diff}")
        pos = comp.cache_pos[:, t * b_t:(t + 1) * b_t]
        assert torch.equal(comp.k_cache[:, t * b_t:(t + 1) * b_t], torch.gather(dev["k"], 1, pos[:, :, None].expand(-1, -1, wl.head_dim)))


@pytest.mark.parametrize("shift", [7, 40, 300])
def test_window_positions_beyond_the_block(shift):
    """Explicit window positions: a window that straddles the end of the block or lies wholly after it
    (a trailing prompt; or the deferred-tail reading of the look-back, where a block's candidates end
    `shift` tokens before its window does).  The causal mask then hides fewer keys, or none."""
    wl = synth.shrink(synth.WORKLOADS["llama8b-16k"], index=14, l_ctx=2048)
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    parts = O.partition(B, wl.n_div, wl.alpha, wl.s_block)
    data = synth.make_layer(wl, 1, parts[0], n_blocks=1)
    dev = to_dev(data)
    s = wl.s_block
    lib = binding.LaserKV(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.dtype, wl.lsh_tables, wl.lsh_bits,
                          max_block=s, max_window=wl.window, max_ctx_keys=0)
    block_pos0 = 5000
    q_pos0 = block_pos0 + s - wl.window + shift
    dbg = dbg_buffers(wl, s)
    keep = torch.empty(wl.n_kv_heads, sum(parts), dtype=torch.int32, device=DEV)
    lib.laserkv_select_block(dev["q_win"][0], dev["k"][:, :s], None, dev["planes"], block_pos0=block_pos0, q_pos0=q_pos0,
                             n_anchor=parts[0], n_local=parts[1], k_exact=parts[2], k_lsh=parts[3], keep_idx=keep,
                             dbg_s_exact=dbg["s_exact"], dbg_sig_k=dbg["sig_k"], dbg_sig_q=dbg["sig_q"], dbg_count=dbg["cnt"])
    torch.cuda.synchronize()
    st = O.select_block(f64(data["q_win"][0]), f64(data["k"][:, :s]), None, f64(data["planes"]), wl.lsh_tables,
                        wl.lsh_bits, *parts, block_pos0=block_pos0, q_pos0=q_pos0)
    rep = check_block(st, gpu_stage(dbg, keep), parts, wl.dtype)
    say(f"[window shift {shift}] max score err/(s+s_k) {rep['max_rel']:.2e}, tolerated {rep['tolerated']}")
    # the last keys of the block are visible to more queries than with the default window
    base = O.exact_scores(f64(data["q_win"][0]), f64(data["k"][:, :s]), None, block_pos0=block_pos0)
    assert (st["s_exact"][:, -1] > base[:, -1]).all()


@pytest.mark.parametrize("name,kw,tail", [("tiny", dict(l_ctx=2048), 40), ("llama8b-16k", dict(l_ctx=8192), 96),
                                          ("llama8b-16k", dict(l_ctx=6144), 0)])
def test_deferred_tail_layer_against_oracle(name, kw, tail):
    """The look-back of Sec. 3.2 read as deferring a block's last `tail` tokens to the next block's call:
    the driver's segment loop (pointer arithmetic into the resident tensors) against the oracle's
    compress_layer_deferred, every segment stage by stage, and the final cache."""
    wl = synth.shrink(synth.WORKLOADS[name], index=19, **kw)
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    na_full = O.partition(B, wl.n_div, wl.alpha, wl.s_block)[0]
    data = synth.make_layer(wl, 2, na_full)
    dev = to_dev(data)
    nb, s = data["q_win"].shape[0], wl.s_block
    comp = LayerCompressor(wl, DEV, tail=tail)
    saved = {}

    def dbg_for(t, seg_len):
        dbg = dbg_buffers(wl, seg_len)
        keep = torch.empty(wl.n_kv_heads, sum(O.partition(B, wl.n_div, wl.alpha, seg_len)), dtype=torch.int32, device=DEV)
        saved[t] = (dbg, keep)
        return dbg, keep

    segs = comp.run_layer_deferred(dev, dbg_for=dbg_for)
    torch.cuda.synchronize()
    k64, v64, q64 = f64(data["k"]), f64(data["v"]), f64(data["q_win"])
    blocks = [(q64[t], k64[:, t * s:(t + 1) * s], v64[:, t * s:(t + 1) * s], t * s) for t in range(nb)]
    cap = sum(min(B, hi - lo) for lo, hi, _, _ in segs)
    ck, cv, cp, clen, stages = O.compress_layer_deferred(blocks, f64(data["planes"]), wl.lsh_tables, wl.lsh_bits, B,
                                                         wl.n_div, wl.alpha, cap=cap, tail=tail)
    assert comp.cache_len == clen == cap
    n_tol = 0
    for t, (lo, hi, n_ctx, keep) in enumerate(segs):
        assert (lo, hi - lo) == (stages[t]["seg_pos0"], stages[t]["seg_len"])
        parts = O.partition(B, wl.n_div, wl.alpha, hi - lo)
        # the oracle's stage used ITS cache rows as look-back keys; they are the raw keys before the segment
        rep = check_block(stages[t], gpu_stage(*saved[t]), parts, wl.dtype)
        n_tol += sum(c for _, c in rep["tolerated"])
    say(f"[deferred-tail {wl.name} tail {tail}] {len(segs)} segments, tolerated index diffs {n_tol}")
    pos = comp.cache_pos[:, :clen]
    assert bool((pos[:, 1:] > pos[:, :-1]).all())
    assert torch.equal(comp.k_cache[:, :clen], torch.gather(dev["k"], 1, pos[:, :, None].expand(-1, -1, wl.head_dim)))
    assert torch.equal(comp.v_cache[:, :clen], torch.gather(dev["v"], 1, pos[:, :, None].expand(-1, -1, wl.head_dim)))
    if n_tol == 0:
        assert np.array_equal(pos.cpu().numpy(), cp[:, :clen])


def test_layers_with_their_own_budgets_share_one_context():
    """A per-layer budget schedule (a pyramid over depth, say) is a host-side choice of the four integers of
    every call: two layers with different B run through ONE library context and each matches the oracle run
    with its own budget."""
    wl = synth.shrink(synth.WORKLOADS["llama8b-16k"], index=20, l_ctx=6144)
    B0 = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    budgets = [B0, B0 // 3]
    shared = None
    for layer, B in enumerate(budgets):
        parts = O.partition(B, wl.n_div, wl.alpha, wl.s_block)
        data = synth.make_layer(wl, layer, parts[0])
        dev = to_dev(data)
        comp = LayerCompressor(wl, DEV, budget=B, lib=shared)
        shared = comp.lib
        nb, s = data["q_win"].shape[0], wl.s_block
        prev_local, saved = 0, []
        for t in range(nb):
            dbg = dbg_buffers(wl, s)
            keep = torch.empty(wl.n_kv_heads, sum(parts), dtype=torch.int32, device=DEV)
            n_ctx = prev_local
            prev_local, _ = comp.step(dev["q_win"][t], dev["k"][:, t * s:(t + 1) * s], dev["v"][:, t * s:(t + 1) * s],
                                      dev["planes"], t * s, prev_local, dbg=dbg, keep_out=keep)
            saved.append((dbg, keep, n_ctx))
        torch.cuda.synchronize()
        assert comp.cache_len == nb * sum(parts) == nb * B
        k64 = f64(data["k"])
        for t, (dbg, keep, n_ctx) in enumerate(saved):
            lo = t * s
            st = O.select_block(f64(data["q_win"][t]), k64[:, lo:lo + s], k64[:, lo - n_ctx:lo] if n_ctx else None,
                                f64(data["planes"]), wl.lsh_tables, wl.lsh_bits, *parts, block_pos0=lo)
            check_block(st, gpu_stage(dbg, keep), parts, wl.dtype)
        say(f"[per-layer budget] layer {layer} B={B} parts={parts}: {nb} blocks match the oracle")


@pytest.mark.parametrize("dtype,window", [("bf16", 40), ("f32", 40), ("bf16", 1)])
def test_padded_query_and_key_strides(dtype, window):
    """Window queries whose head stride is not W rows (a slice of a longer tensor) and keys whose row stride
    exceeds head_dim (a slice of a wider tensor): the general addressing paths of the sweeps' load phase.
    A window of one query exercises row / W with W = 1."""
    wl = synth.shrink(synth.WORKLOADS["llama8b-16k"], index=25, l_ctx=2048, s_block=1024, dtype=dtype, window=window)
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    parts = O.partition(B, wl.n_div, wl.alpha, wl.s_block)
    data = synth.make_layer(wl, 0, parts[0], n_blocks=1)
    s, d, w = wl.s_block, wl.head_dim, wl.window
    q_pad = torch.zeros(wl.n_q_heads, w + 5, d, dtype=wl.torch_dtype, device=DEV)
    q_pad[:, 2:2 + w] = data["q_win"][0].to(DEV)
    k_wide = torch.zeros(wl.n_kv_heads, s, d + 64, dtype=wl.torch_dtype, device=DEV)
    k_wide[:, :, 8:8 + d] = data["k"][:, :s].to(DEV)
    q_view, k_view = q_pad[:, 2:2 + w], k_wide[:, :, 8:8 + d]
    assert q_view.stride(0) != w * q_view.stride(1) and k_view.stride(1) == d + 64
    lib = binding.LaserKV(wl.n_q_heads, wl.n_kv_heads, d, wl.dtype, wl.lsh_tables, wl.lsh_bits,
                          max_block=s, max_window=w, max_ctx_keys=0)
    dbg = dbg_buffers(wl, s)
    keep = torch.empty(wl.n_kv_heads, sum(parts), dtype=torch.int32, device=DEV)
    lib.laserkv_select_block(q_view, k_view, None, data["planes"].to(DEV), block_pos0=0,
                             n_anchor=parts[0], n_local=parts[1], k_exact=parts[2], k_lsh=parts[3], keep_idx=keep,
                             dbg_s_exact=dbg["s_exact"], dbg_sig_k=dbg["sig_k"], dbg_sig_q=dbg["sig_q"], dbg_count=dbg["cnt"])
    torch.cuda.synchronize()
    st = O.select_block(f64(data["q_win"][0]), f64(data["k"][:, :s]), None, f64(data["planes"]), wl.lsh_tables,
                        wl.lsh_bits, *parts, block_pos0=0)
    rep = check_block(st, gpu_stage(dbg, keep), parts, wl.dtype)
    say(f"[padded strides {dtype}] max score err/(s+s_k) {rep['max_rel']:.2e}, tolerated {rep['tolerated']}")
    lib.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_query_heads_that_alias_one_tensor(dtype):
    """Every query head reads the same window rows (head stride 0, as an expanded tensor has): no single buffer
    descriptor covers a group whose heads overlap, so the sweeps take their per-row addressing path."""
    wl = synth.shrink(synth.WORKLOADS["llama8b-16k"], index=27, l_ctx=2048, s_block=1024, dtype=dtype)
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    parts = O.partition(B, wl.n_div, wl.alpha, wl.s_block)
    data = synth.make_layer(wl, 0, parts[0], n_blocks=1)
    s, d, w = wl.s_block, wl.head_dim, wl.window
    q_one = data["q_win"][0][3:4].contiguous()
    q_view = q_one.to(DEV).expand(wl.n_q_heads, w, d)
    assert q_view.stride(0) == 0
    lib = binding.LaserKV(wl.n_q_heads, wl.n_kv_heads, d, wl.dtype, wl.lsh_tables, wl.lsh_bits,
                          max_block=s, max_window=w, max_ctx_keys=0)
    dbg = dbg_buffers(wl, s)
    keep = torch.empty(wl.n_kv_heads, sum(parts), dtype=torch.int32, device=DEV)
    lib.laserkv_select_block(q_view, data["k"][:, :s].to(DEV), None, data["planes"].to(DEV), block_pos0=0,
                             n_anchor=parts[0], n_local=parts[1], k_exact=parts[2], k_lsh=parts[3], keep_idx=keep,
                             dbg_s_exact=dbg["s_exact"], dbg_sig_k=dbg["sig_k"], dbg_sig_q=dbg["sig_q"], dbg_count=dbg["cnt"])
    torch.cuda.synchronize()
    st = O.select_block(f64(q_one.expand(wl.n_q_heads, w, d)), f64(data["k"][:, :s]), None, f64(data["planes"]), wl.lsh_tables,
                        wl.lsh_bits, *parts, block_pos0=0)
    rep = check_block(st, gpu_stage(dbg, keep), parts, wl.dtype)
    say(f"[aliased query heads {dtype}] max score err/(s+s_k) {rep['max_rel']:.2e}, tolerated {rep['tolerated']}")
    lib.close()


@pytest.mark.parametrize("s_t,t_ctx,dtype", [(96, 700, "bf16"), (40, 333, "f32"), (1024, 31, "bf16")])
def test_look_back_keys_outnumbering_the_block(s_t, t_ctx, dtype):
    """Look-back keys are spread evenly over the block's key ranges; when there are far more of them than
    block keys, further ranges hold look-back keys only.  Scores must still carry their full weight."""
    wl = synth.shrink(synth.WORKLOADS["llama8b-16k"], index=27, l_ctx=2 * s_t, s_block=s_t, dtype=dtype, window=8,
                      n_q_heads=8, n_kv_heads=2)
    parts = O.partition(s_t // 2, wl.n_div, wl.alpha, s_t)
    data = synth.make_layer(wl, 0, parts[0], n_blocks=1)
    gen = torch.Generator().manual_seed(99)
    k_ctx = (torch.randn(wl.n_kv_heads, t_ctx, wl.head_dim, generator=gen) * 1.2).to(wl.torch_dtype)
    lib = binding.LaserKV(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.dtype, wl.lsh_tables, wl.lsh_bits,
                          max_block=s_t, max_window=wl.window, max_ctx_keys=t_ctx)
    dbg = dbg_buffers(wl, s_t)
    keep = torch.empty(wl.n_kv_heads, sum(parts), dtype=torch.int32, device=DEV)
    lib.laserkv_select_block(data["q_win"][0].to(DEV), data["k"][:, :s_t].to(DEV), k_ctx.to(DEV), data["planes"].to(DEV),
                             block_pos0=4096, n_anchor=parts[0], n_local=parts[1], k_exact=parts[2], k_lsh=parts[3],
                             keep_idx=keep, dbg_s_exact=dbg["s_exact"], dbg_sig_k=dbg["sig_k"], dbg_sig_q=dbg["sig_q"],
                             dbg_count=dbg["cnt"])
    torch.cuda.synchronize()
    st = O.select_block(f64(data["q_win"][0]), f64(data["k"][:, :s_t]), f64(k_ctx), f64(data["planes"]), wl.lsh_tables,
                        wl.lsh_bits, *parts, block_pos0=4096)
    rep = check_block(st, gpu_stage(dbg, keep), parts, wl.dtype)
    say(f"[look-back {t_ctx} keys, block {s_t}, {dtype}] max score err/(s+s_k) {rep['max_rel']:.2e}, tolerated {rep['tolerated']}")
    if t_ctx > s_t:
        assert st["s_exact"].sum(1).max() < 0.9  # the look-back keys hold a real share of the mass
    lib.close()
