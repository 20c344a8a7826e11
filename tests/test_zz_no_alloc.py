"""laserkv_compress_block_static (the entry point that allocates nothing) against laserkv_compress_block:
two calls in a row through the C-ABI, the second with a smaller input, bit-identical outputs."""
import pytest
import torch

from oracle import laserkv_oracle as O
from paper_2602_02199_amd import binding, synth

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _run_both(wl, layer, n_blocks, s_t=None):
    """One layer prefix through both entry points; returns the two (keep per block, cache) results."""
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    s = wl.s_block if s_t is None else s_t
    parts = O.partition(B, wl.n_div, wl.alpha, s)
    na, nl, ke, kl = parts
    b_t = sum(parts)
    data = synth.make_layer(wl, layer, O.partition(B, wl.n_div, wl.alpha, wl.s_block)[0], n_blocks=n_blocks)
    dev = {k: v.to(DEV) for k, v in data.items() if k != "needles"}
    cfg = binding.Config(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, binding.LKV_BF16 if wl.dtype == "bf16" else binding.LKV_F32,
                         wl.lsh_tables, wl.lsh_bits, wl.s_block, wl.window, nl)
    assert 0 < binding.laserkv_static_workspace_bytes(cfg) <= binding.LKV_STATIC_SCRATCH_BYTES
    lib = binding.LaserKV(wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.dtype, wl.lsh_tables, wl.lsh_bits,
                          max_block=wl.s_block, max_window=wl.window, max_ctx_keys=nl)
    stream = torch.cuda.current_stream().cuda_stream
    results = []
    for static in (False, True):
        cap = n_blocks * b_t
        kc = torch.zeros(wl.n_kv_heads, cap, wl.head_dim, dtype=wl.torch_dtype, device=DEV)
        vc = torch.zeros_like(kc)
        pos = torch.full((wl.n_kv_heads, cap), -1, dtype=torch.int64, device=DEV)
        keeps = []
        for t in range(n_blocks):
            lo = t * wl.s_block
            keep = torch.full((wl.n_kv_heads, b_t), -1, dtype=torch.int32, device=DEV)
            k_ctx = kc[:, t * b_t - nl:t * b_t] if t else None
            kw = dict(block_pos0=lo, n_anchor=na, n_local=nl, k_exact=ke, k_lsh=kl, keep_idx=keep, k_cache=kc, v_cache=vc,
                      cache_pos=pos, cache_len=t * b_t)
            args = (dev["q_win"][t], dev["k"][:, lo:lo + s], dev["v"][:, lo:lo + s], k_ctx, dev["planes"])
            if static:
                binding.laserkv_compress_block_static(cfg, *args, stream=stream, **kw)
            else:
                lib.laserkv_compress_block(*args, **kw)
            keeps.append(keep)
        torch.cuda.synchronize()
        results.append((torch.stack(keeps), kc, vc, pos))
    lib.close()
    return results


def test_static_entry_point_matches_compress_block_on_consecutive_calls():
    print("[no-alloc] set-up of the static scratch on cuda:0", flush=True)
    binding.laserkv_static_init()
    # first a large input (every block of a 16k layer, 8 heads x 2048 keys), then a smaller one (fp32, 2 heads
    # x 512 keys, then a ragged block length) on the same scratch array
    cases = [(synth.WORKLOADS["llama8b-16k"], 1, 3, None),
             (synth.WORKLOADS["tiny"], 2, 2, None),
             (synth.shrink(synth.WORKLOADS["tiny"], index=31, l_ctx=1024), 0, 2, 333),
             (synth.WORKLOADS["llama8b-128k"], 0, 2, None)]
    for wl, layer, nb, s_t in cases:
        print(f"[no-alloc] {wl.name} layer {layer}, {nb} blocks, s_t {s_t or wl.s_block}", flush=True)
        ref, got = _run_both(wl, layer, nb, s_t)
        for a, b in zip(ref, got):
            assert torch.equal(a, b)
        assert bool((ref[0] >= 0).all())


def test_static_entry_point_rejects_what_does_not_fit():
    cfg = binding.Config(64, 64, 128, binding.LKV_BF16, 32, 12, 16384, 16, 4096)
    assert binding.laserkv_static_workspace_bytes(cfg) > binding.LKV_STATIC_SCRATCH_BYTES
    q = torch.zeros(64, 16, 128, dtype=torch.bfloat16, device=DEV)
    k = torch.zeros(64, 64, 128, dtype=torch.bfloat16, device=DEV)
    planes = torch.zeros(384, 128, dtype=torch.bfloat16, device=DEV)
    keep = torch.full((64, 8), -7, dtype=torch.int32, device=DEV)
    pos = torch.zeros(64, 64, dtype=torch.int64, device=DEV)
    with pytest.raises(binding.LaserKVError) as ei:
        binding.laserkv_compress_block_static(cfg, q, k, k, None, planes, block_pos0=0, n_anchor=2, n_local=2, k_exact=2,
                                              k_lsh=2, keep_idx=keep, k_cache=k.clone(), v_cache=k.clone(), cache_pos=pos,
                                              cache_len=0, stream=torch.cuda.current_stream().cuda_stream)
    assert ei.value.code == binding.LKV_EINVAL and "static" in str(ei.value)
    torch.cuda.synchronize()
    assert bool((keep == -7).all())
