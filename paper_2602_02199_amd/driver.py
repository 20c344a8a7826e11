"""Block loop of one layer on the GPU: the sequence of library calls a prefill engine makes.

For every context block (Sec. 3.2) it calls laserkv_select_block and laserkv_append on the
current stream without any host synchronisation: each block adds exactly B_t rows per head, so
cache lengths are known on the host.  Look-back keys of block t are the previous block's local
window, i.e. the last n_local rows already in the cache (passed as a strided view, no copy).
"""
from __future__ import annotations

import torch

from . import binding


class LayerCompressor:
    def __init__(self, wl, device="cuda:0", max_blocks=None, budget=None, tail=0, lib=None):
        """budget: per-block budget B of this layer (default: the App. B equation for the workload; a
        per-layer schedule passes its own).  tail: tokens a block defers to the next one (run_layer_deferred);
        blocks handed to the library are then up to s_block + tail long.  lib: an existing library context
        of sufficient limits to share (its workspace does not depend on the budget)."""
        self.wl = wl
        self.device = torch.device(device)
        self.B = binding.laserkv_budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den) if budget is None else int(budget)
        self.parts = binding.laserkv_partition(self.B, wl.n_div, wl.alpha, wl.s_block)
        nb = wl.n_blocks if max_blocks is None else max_blocks
        self.tail = int(tail)
        self.cap = nb * min(self.B, wl.s_block + self.tail)
        max_local = binding.laserkv_partition(self.B, wl.n_div, wl.alpha, wl.s_block + self.tail)[1]
        self.lib = lib if lib is not None else binding.LaserKV(
            wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.dtype, wl.lsh_tables, wl.lsh_bits,
            max_block=wl.s_block + self.tail, max_window=wl.window, max_ctx_keys=max_local)
        dt = wl.torch_dtype
        self.k_cache = torch.zeros(wl.n_kv_heads, self.cap, wl.head_dim, dtype=dt, device=self.device)
        self.v_cache = torch.zeros_like(self.k_cache)
        self.cache_pos = torch.full((wl.n_kv_heads, self.cap), -1, dtype=torch.int64, device=self.device)
        self.keep = torch.empty(wl.n_kv_heads, min(self.B, wl.s_block), dtype=torch.int32, device=self.device)
        self.cache_len = 0

    def reset(self):
        self.cache_len = 0

    def run_layer_deferred(self, data, n_blocks=None, dbg_for=None):
        """The layer loop with each block's last `tail` tokens deferred to the next block's call (the look-back
        of Sec. 3.2 read as judging a block's edge only once later context exists): call t covers positions
        [block start - tail, block end - tail) (the first starts with its block, the last ends with its block)
        and is scored by the block's own last W tokens at their real positions.  Pointer arithmetic only.

        dbg_for: optional callable(t, seg_len) -> (dbg dict or None, keep tensor or None) supplying stage-output
        buffers for segment t.  Returns [(seg_lo, seg_hi, n_ctx, keep)] per segment."""
        wl, tail = self.wl, self.tail
        self.reset()
        nb = data["q_win"].shape[0] if n_blocks is None else n_blocks
        l_tot = data["k"].shape[1]
        prev_local, out = 0, []
        for t in range(nb):
            blk_lo, blk_hi = t * wl.s_block, min((t + 1) * wl.s_block, l_tot)
            lo = blk_lo - (tail if t else 0)
            hi = blk_hi - (tail if t < nb - 1 else 0)
            na, nl, ke, kl = binding.laserkv_partition(self.B, wl.n_div, wl.alpha, hi - lo)
            b_t = na + nl + ke + kl
            dbg, keep = dbg_for(t, hi - lo) if dbg_for else (None, None)
            if keep is None:
                keep = torch.empty(wl.n_kv_heads, b_t, dtype=torch.int32, device=self.device)
            dbg = dbg or {}
            k_ctx = self.k_cache[:, self.cache_len - prev_local:self.cache_len] if (self.cache_len and prev_local) else None
            k_seg, v_seg = data["k"][:, lo:hi], data["v"][:, lo:hi]
            self.lib.laserkv_select_block(data["q_win"][t], k_seg, k_ctx, data["planes"], block_pos0=lo,
                                          q_pos0=blk_hi - wl.window, causal=True,
                                          n_anchor=na, n_local=nl, k_exact=ke, k_lsh=kl, keep_idx=keep,
                                          dbg_s_exact=dbg.get("s_exact"), dbg_sig_k=dbg.get("sig_k"),
                                          dbg_sig_q=dbg.get("sig_q"), dbg_count=dbg.get("cnt"))
            self.lib.laserkv_append(k_seg, v_seg, keep, b_t=b_t, block_pos0=lo, k_cache=self.k_cache,
                                    v_cache=self.v_cache, cache_pos=self.cache_pos, cache_len=self.cache_len)
            self.cache_len += b_t
            out.append((lo, hi, prev_local, keep))
            prev_local = nl
        return out

    def block_budget(self, s_t):
        """(n_anchor, n_local, k_exact, k_lsh) of a block with s_t tokens."""
        if s_t == self.wl.s_block:
            return self.parts
        return binding.laserkv_partition(self.B, self.wl.n_div, self.wl.alpha, s_t)

    def step(self, q_win, k_blk, v_blk, planes, block_pos0, prev_local, dbg=None, keep_out=None):
        """One block: select + append.  Returns (this block's n_local, the keep tensor used).

        keep_out: optional [H_kv, B_t] int32 device tensor to receive the kept indices (the internal
        buffer is reused from block to block otherwise).  dbg: optional dict of device tensors for the
        stage outputs (s_exact, sig_k, sig_q, cnt).
        """
        s_t = k_blk.shape[1]
        na, nl, ke, kl = self.block_budget(s_t)
        b_t = na + nl + ke + kl
        k_ctx = None
        if self.cache_len and prev_local:
            k_ctx = self.k_cache[:, self.cache_len - prev_local:self.cache_len]
        if keep_out is not None:
            keep = keep_out
        elif b_t == self.keep.shape[1]:
            keep = self.keep
        else:
            keep = torch.empty(self.wl.n_kv_heads, b_t, dtype=torch.int32, device=self.device)
        assert keep.shape == (self.wl.n_kv_heads, b_t) and keep.is_contiguous()
        dbg = dbg or {}
        self.lib.laserkv_select_block(q_win, k_blk, k_ctx, planes, block_pos0=block_pos0, causal=True,
                                      n_anchor=na, n_local=nl, k_exact=ke, k_lsh=kl, keep_idx=keep,
                                      dbg_s_exact=dbg.get("s_exact"), dbg_sig_k=dbg.get("sig_k"),
                                      dbg_sig_q=dbg.get("sig_q"), dbg_count=dbg.get("cnt"))
        self.lib.laserkv_append(k_blk, v_blk, keep, b_t=b_t, block_pos0=block_pos0, k_cache=self.k_cache,
                                v_cache=self.v_cache, cache_pos=self.cache_pos, cache_len=self.cache_len)
        self.cache_len += b_t
        return nl, keep

    def run_layer(self, data, n_blocks=None):
        """All blocks of one layer, back to back, no host sync.  data: device tensors from synth.make_layer."""
        wl = self.wl
        self.reset()
        nb = data["q_win"].shape[0] if n_blocks is None else n_blocks
        prev_local = 0
        l_tot = data["k"].shape[1]
        for t in range(nb):
            lo, hi = t * wl.s_block, min((t + 1) * wl.s_block, l_tot)
            prev_local, _ = self.step(data["q_win"][t], data["k"][:, lo:hi], data["v"][:, lo:hi], data["planes"],
                                      lo, prev_local)
        return self.cache_len

    def run_layer_with_attention(self, data, q_blocks, out, lse, lse_win, workspace, n_blocks=None):
        """The block loop as a model runs it (Sec. 3 first paragraph; Sec. 3.3 "Precision"): block t's queries
        attend to the compacted cache and, causally, to the block itself (laserkv_attend_block); the window
        rows' log-sum-exp that kernel reports is handed to the selection as the complete row statistic
        (laserkv_set_row_lse_complete: one sweep over the block, no statistics of its own); the kept rows join
        the cache the next block attends to.  No host synchronisation.

        q_blocks[t]: [H_q, S_t, d] queries of block t, whose last W rows are the observation window (passed to
        the selection as a view).  out [H_q, S, d] and lse [H_q, S] float32 receive each block's attention,
        lse_win [H_q, W] float32 the window rows' statistics, workspace the attention scratch (sized for the
        last block); all are reused from block to block."""
        wl = self.wl
        self.reset()
        nb = len(q_blocks) if n_blocks is None else n_blocks
        l_tot = data["k"].shape[1]
        w = wl.window
        for t in range(nb):
            lo, hi = t * wl.s_block, min((t + 1) * wl.s_block, l_tot)
            s_t = hi - lo
            q, k_blk, v_blk = q_blocks[t], data["k"][:, lo:hi], data["v"][:, lo:hi]
            # contiguous [H_q, s_t, ...] tensors at the start of the buffers (a short last block uses less of them)
            out_now = out.view(-1)[:q.shape[0] * s_t * wl.head_dim].view(q.shape[0], s_t, wl.head_dim)
            lse_now = lse.view(-1)[:q.shape[0] * s_t].view(q.shape[0], s_t)
            self.lib.laserkv_attend_block(q, self.k_cache, self.v_cache, k_blk, v_blk, cache_len=self.cache_len, block_pos0=lo,
                                          out=out_now, out_lse=lse_now, workspace=workspace)
            lse_win.copy_(lse_now[:, s_t - w:])
            self.lib.laserkv_set_row_lse_complete(lse_win)
            na, nl, ke, kl = self.block_budget(s_t)
            b_t = na + nl + ke + kl
            keep = self.keep if b_t == self.keep.shape[1] else torch.empty(wl.n_kv_heads, b_t, dtype=torch.int32, device=self.device)
            self.lib.laserkv_compress_block(q[:, s_t - w:], k_blk, v_blk, None, data["planes"], block_pos0=lo, n_anchor=na,
                                            n_local=nl, k_exact=ke, k_lsh=kl, keep_idx=keep, k_cache=self.k_cache,
                                            v_cache=self.v_cache, cache_pos=self.cache_pos, cache_len=self.cache_len)
            self.cache_len += b_t
        self.lib.laserkv_set_row_lse_complete(None)
        return self.cache_len

    # ---- pre-marshalled call lists: one ctypes call per library entry point, nothing else ----
    def plan_layer(self, data, n_blocks=None, fused=True, row_lse_complete=None):
        """Builds the layer's call list once: [(c_function, argument tuple without the stream)].

        The tensors in `data`, the cache and the keep buffer must stay alive and in place while the
        plan is used.  run_plan() then issues the calls back to back with no per-call Python work
        beyond the foreign call itself (and can be captured into a HIP graph).  fused=True uses
        laserkv_compress_block (one call per block), else laserkv_select_block + laserkv_append.
        row_lse_complete: optional list of per-block float32 [H_q, W] device tensors with the window rows'
        complete log-sum-exp (what the model's attention kernel reports); each block's call is then preceded
        by laserkv_set_row_lse_complete, and look-back keys are not passed.
        """
        import ctypes as C
        wl, lib = self.wl, self.lib._lib
        ctx = self.lib._ctx
        vp = C.c_void_p
        nb = data["q_win"].shape[0] if n_blocks is None else n_blocks
        l_tot = data["k"].shape[1]
        d = wl.head_dim
        calls, cache_len, prev_local = [], 0, 0
        kc_sh, kc_st = self.k_cache.stride(0), self.k_cache.stride(1)
        es = self.k_cache.element_size()
        for t in range(nb):
            lo, hi = t * wl.s_block, min((t + 1) * wl.s_block, l_tot)
            s_t = hi - lo
            na, nl, ke, kl = self.block_budget(s_t)
            b_t = na + nl + ke + kl
            assert b_t == self.keep.shape[1], "plans cover equal-sized blocks only"
            q, k, v = data["q_win"][t], data["k"][:, lo:hi], data["v"][:, lo:hi]
            t_ctx = prev_local if cache_len else 0
            if row_lse_complete is not None:
                lse = row_lse_complete[t]
                assert lse.is_contiguous() and lse.dtype == torch.float32 and lse.shape == (wl.n_q_heads, wl.window)
                calls.append((lib.laserkv_set_row_lse_complete, (ctx, vp(lse.data_ptr())), False))
                t_ctx = 0
            ctx_ptr = vp(self.k_cache.data_ptr() + (cache_len - t_ctx) * kc_st * es) if t_ctx else None
            if fused:
                calls.append((lib.laserkv_compress_block, (
                    ctx, vp(q.data_ptr()), q.stride(0), q.stride(1), vp(k.data_ptr()), k.stride(0), k.stride(1),
                    vp(v.data_ptr()), v.stride(0), v.stride(1),
                    ctx_ptr, kc_sh if t_ctx else 0, kc_st if t_ctx else 0, vp(data["planes"].data_ptr()),
                    s_t, wl.window, t_ctx, lo, binding.LKV_WINDOW_AT_BLOCK_END, 1, na, nl, ke, kl,
                    vp(self.keep.data_ptr()), vp(self.k_cache.data_ptr()), vp(self.v_cache.data_ptr()), kc_sh,
                    vp(self.cache_pos.data_ptr()), self.cache_pos.stride(0), cache_len, self.cap), True))
            else:
                calls.append((lib.laserkv_select_block, (
                    ctx, vp(q.data_ptr()), q.stride(0), q.stride(1), vp(k.data_ptr()), k.stride(0), k.stride(1),
                    ctx_ptr, kc_sh if t_ctx else 0, kc_st if t_ctx else 0, vp(data["planes"].data_ptr()),
                    s_t, wl.window, t_ctx, lo, binding.LKV_WINDOW_AT_BLOCK_END, 1, na, nl, ke, kl,
                    vp(self.keep.data_ptr()), None, None, None, None), True))
                calls.append((lib.laserkv_append, (
                    ctx, vp(k.data_ptr()), k.stride(0), k.stride(1), vp(v.data_ptr()), v.stride(0), v.stride(1),
                    vp(self.keep.data_ptr()), b_t, s_t, lo, vp(self.k_cache.data_ptr()), vp(self.v_cache.data_ptr()),
                    kc_sh, vp(self.cache_pos.data_ptr()), self.cache_pos.stride(0), cache_len, self.cap), True))
            cache_len += b_t
            prev_local = nl
        if row_lse_complete is not None:   # leave the context computing its own statistics again
            calls.append((lib.laserkv_set_row_lse_complete, (ctx, None), False))
        self._plan_len = cache_len
        return calls

    def run_plan(self, calls, stream=None):
        import ctypes as C
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        sp = C.c_void_p(stream)
        for fn, args, takes_stream in calls:
            rc = fn(*args, sp) if takes_stream else fn(*args)
            if rc != 0:
                self.lib._check(rc)
        self.cache_len = self._plan_len
        return self.cache_len
