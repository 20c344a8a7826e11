"""Thin ctypes binding of liblaserkv.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels.  There is no CPU
fallback: loading fails loudly when the library has not been built.
PyTorch is used by callers for device memory and streams; this module only
reads `data_ptr()`, strides and the current stream handle.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "liblaserkv.so")

LKV_F32, LKV_BF16 = 0, 1
LKV_OK, LKV_EINVAL, LKV_ECAP, LKV_ENOMEM, LKV_EHIP = 0, -1, -2, -3, -4
LKV_WINDOW_AT_BLOCK_END = -(1 << 63)   # q_pos0 sentinel of laserkv.h

EXPORTS = (
    "laserkv_create", "laserkv_destroy", "laserkv_last_error", "laserkv_budget",
    "laserkv_partition", "laserkv_select_block", "laserkv_append", "laserkv_compress_block",
    "laserkv_profile_begin", "laserkv_profile_end", "laserkv_profile_isolate",
    "laserkv_score_block", "laserkv_select_consensus", "laserkv_append_shared", "laserkv_set_row_lse",
    "laserkv_set_row_lse_complete", "laserkv_attend_workspace_bytes", "laserkv_attend_cache",
    "laserkv_attend_block_workspace_bytes", "laserkv_attend_block",
    "laserkv_static_init", "laserkv_static_workspace_bytes", "laserkv_compress_block_static",
)
LKV_STATIC_SCRATCH_BYTES = 32 << 20
KERNEL_NAMES = ("sweep1", "sweep2", "count", "select", "append", "attend", "single")


class LaserKVError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"laserkv error {code}: {msg}")
        self.code = code


class Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in (
        "n_q_heads", "n_kv_heads", "head_dim", "dtype", "lsh_tables", "lsh_bits",
        "max_block", "max_window", "max_ctx_keys")]


_lib = None


def load():
    """Load the built library (never builds, never falls back)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is missing: build it first with `python -m paper_2602_02199_amd.build` "
            "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, i64 = C.c_void_p, C.c_int32, C.c_int64
    lib.laserkv_create.argtypes = [C.POINTER(Config), C.POINTER(vp)]
    lib.laserkv_create.restype = C.c_int
    lib.laserkv_destroy.argtypes = [vp]
    lib.laserkv_destroy.restype = None
    lib.laserkv_last_error.argtypes = [vp]
    lib.laserkv_last_error.restype = C.c_char_p
    lib.laserkv_budget.argtypes = [i64, i64, i64, i64]
    lib.laserkv_budget.restype = i64
    lib.laserkv_partition.argtypes = [i32, i32, C.c_double, i32] + [C.POINTER(i32)] * 4
    lib.laserkv_partition.restype = C.c_int
    lib.laserkv_select_block.argtypes = [
        vp, vp, i64, i64, vp, i64, i64, vp, i64, i64, vp,
        i32, i32, i32, i64, i64, i32, i32, i32, i32, i32,
        vp, vp, vp, vp, vp, vp]
    lib.laserkv_select_block.restype = C.c_int
    lib.laserkv_append.argtypes = [
        vp, vp, i64, i64, vp, i64, i64, vp, i32, i32, i64,
        vp, vp, i64, vp, i64, i64, i64, vp]
    lib.laserkv_append.restype = C.c_int
    lib.laserkv_compress_block.argtypes = [
        vp, vp, i64, i64, vp, i64, i64, vp, i64, i64, vp, i64, i64, vp,
        i32, i32, i32, i64, i64, i32, i32, i32, i32, i32,
        vp, vp, vp, i64, vp, i64, i64, i64, vp]
    lib.laserkv_compress_block.restype = C.c_int
    lib.laserkv_static_init.argtypes = []
    lib.laserkv_static_init.restype = C.c_int
    lib.laserkv_static_workspace_bytes.argtypes = [C.POINTER(Config)]
    lib.laserkv_static_workspace_bytes.restype = C.c_size_t
    lib.laserkv_compress_block_static.argtypes = [C.POINTER(Config)] + lib.laserkv_compress_block.argtypes[1:]
    lib.laserkv_compress_block_static.restype = C.c_int
    lib.laserkv_score_block.argtypes = [
        vp, vp, i64, i64, vp, i64, i64, vp, i64, i64, vp,
        i32, i32, i32, i64, i64, i32, vp, vp, i32, vp]
    lib.laserkv_score_block.restype = C.c_int
    lib.laserkv_select_consensus.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, vp, vp]
    lib.laserkv_select_consensus.restype = C.c_int
    lib.laserkv_append_shared.argtypes = lib.laserkv_append.argtypes
    lib.laserkv_append_shared.restype = C.c_int
    lib.laserkv_set_row_lse.argtypes = [vp, vp]
    lib.laserkv_set_row_lse.restype = C.c_int
    lib.laserkv_set_row_lse_complete.argtypes = [vp, vp]
    lib.laserkv_set_row_lse_complete.restype = C.c_int
    lib.laserkv_attend_workspace_bytes.argtypes = [vp, i32, i64]
    lib.laserkv_attend_workspace_bytes.restype = i64
    lib.laserkv_attend_cache.argtypes = [vp, vp, i64, i64, i32, vp, vp, i64, i64, vp, vp, vp, i64, vp]
    lib.laserkv_attend_cache.restype = C.c_int
    lib.laserkv_attend_block_workspace_bytes.argtypes = [vp, i32, i64, i32]
    lib.laserkv_attend_block_workspace_bytes.restype = i64
    lib.laserkv_attend_block.argtypes = [vp, vp, i64, i64, i32, vp, vp, i64, i64, vp, i64, i64, vp, i64, i64,
                                         i32, i64, i64, i32, vp, vp, vp, i64, vp]
    lib.laserkv_attend_block.restype = C.c_int
    lib.laserkv_profile_begin.argtypes = [vp]
    lib.laserkv_profile_begin.restype = C.c_int
    lib.laserkv_profile_end.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(i64)]
    lib.laserkv_profile_end.restype = C.c_int
    lib.laserkv_profile_isolate.argtypes = [vp, i32]
    lib.laserkv_profile_isolate.restype = C.c_int
    _lib = lib
    return lib


def laserkv_budget(s_block: int, l_ctx: int, r_num: int = 1, r_den: int = 4) -> int:
    b = load().laserkv_budget(s_block, l_ctx, r_num, r_den)
    if b < 0:
        raise LaserKVError(LKV_EINVAL, "budget: bad arguments")
    return int(b)


def laserkv_partition(B: int, n: int, alpha: float, s_t: int):
    lib = load()
    out = [C.c_int32() for _ in range(4)]
    rc = lib.laserkv_partition(B, n, alpha, s_t, *[C.byref(o) for o in out])
    if rc != LKV_OK:
        raise LaserKVError(rc, lib.laserkv_last_error(None).decode())
    return tuple(int(o.value) for o in out)


def laserkv_static_init():
    lib = load()
    rc = lib.laserkv_static_init()
    if rc != LKV_OK:
        raise LaserKVError(rc, lib.laserkv_last_error(None).decode())


def laserkv_static_workspace_bytes(cfg: Config) -> int:
    return int(load().laserkv_static_workspace_bytes(C.byref(cfg)))


def laserkv_compress_block_static(cfg: Config, q_win, k_blk, v_blk, k_ctx, hyperplanes, *, block_pos0, q_pos0=None,
                                  causal=True, n_anchor, n_local, k_exact, k_lsh, keep_idx, k_cache, v_cache, cache_pos,
                                  cache_len, stream):
    """laserkv_compress_block on the library's static scratch (no context, no allocation).  stream: raw handle."""
    lib = load()
    d = cfg.head_dim
    s_t, w = k_blk.shape[1], q_win.shape[1]
    t_ctx = 0 if k_ctx is None else k_ctx.shape[1]
    if q_pos0 is None:
        q_pos0 = LKV_WINDOW_AT_BLOCK_END
    qs, ks, vs = _strides3(q_win, d), _strides3(k_blk, d), _strides3(v_blk, d)
    cs = _strides3(k_ctx, d) if k_ctx is not None else (0, 0)
    assert hyperplanes.is_contiguous()
    assert k_cache.stride(2) == 1 and k_cache.stride(1) == d and v_cache.stride() == k_cache.stride()
    rc = lib.laserkv_compress_block_static(
        C.byref(cfg), _ptr(q_win), qs[0], qs[1], _ptr(k_blk), ks[0], ks[1], _ptr(v_blk), vs[0], vs[1],
        _ptr(k_ctx), cs[0], cs[1], _ptr(hyperplanes), s_t, w, t_ctx, block_pos0, q_pos0, 1 if causal else 0,
        n_anchor, n_local, k_exact, k_lsh, _ptr(keep_idx), _ptr(k_cache), _ptr(v_cache), k_cache.stride(0),
        _ptr(cache_pos), cache_pos.stride(0), cache_len, k_cache.shape[1], C.c_void_p(stream))
    if rc != LKV_OK:
        raise LaserKVError(rc, lib.laserkv_last_error(None).decode())


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _strides3(t, d):
    assert t.dim() == 3 and t.stride(2) == 1 and t.shape[2] == d, "expected [heads, rows, d] with d contiguous"
    return t.stride(0), t.stride(1)


class LaserKV:
    """One library context (owns the device workspace).  Methods mirror the C entry points."""

    def __init__(self, n_q_heads, n_kv_heads, head_dim, dtype, lsh_tables, lsh_bits,
                 max_block, max_window, max_ctx_keys):
        import torch
        self._lib = load()
        self._torch = torch
        if not torch.cuda.is_available():
            raise RuntimeError("laserkv needs a GPU: there is no CPU path")
        self.cfg = Config(n_q_heads, n_kv_heads, head_dim,
                          {"f32": LKV_F32, "bf16": LKV_BF16}[dtype] if isinstance(dtype, str) else dtype,
                          lsh_tables, lsh_bits, max_block, max_window, max_ctx_keys)
        self._ctx = C.c_void_p()
        rc = self._lib.laserkv_create(C.byref(self.cfg), C.byref(self._ctx))
        if rc != LKV_OK:
            raise LaserKVError(rc, self._lib.laserkv_last_error(None).decode())

    def close(self):
        if getattr(self, "_ctx", None) is not None and self._ctx:
            self._lib.laserkv_destroy(self._ctx)
            self._ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc):
        if rc != LKV_OK:
            raise LaserKVError(rc, self._lib.laserkv_last_error(self._ctx).decode())

    def _stream(self, stream):
        if stream is None:
            stream = self._torch.cuda.current_stream().cuda_stream
        return C.c_void_p(stream)

    def laserkv_select_block(self, q_win, k_blk, k_ctx, hyperplanes, *, block_pos0, q_pos0=None, causal=True,
                             n_anchor, n_local, k_exact, k_lsh, keep_idx,
                             dbg_s_exact=None, dbg_sig_k=None, dbg_sig_q=None, dbg_count=None, stream=None):
        d = self.cfg.head_dim
        s_t, w = k_blk.shape[1], q_win.shape[1]
        t_ctx = 0 if k_ctx is None else k_ctx.shape[1]
        if q_pos0 is None:
            q_pos0 = LKV_WINDOW_AT_BLOCK_END
        qs, ks = _strides3(q_win, d), _strides3(k_blk, d)
        cs = _strides3(k_ctx, d) if k_ctx is not None else (0, 0)
        assert hyperplanes.is_contiguous()
        rc = self._lib.laserkv_select_block(
            self._ctx, _ptr(q_win), qs[0], qs[1], _ptr(k_blk), ks[0], ks[1], _ptr(k_ctx), cs[0], cs[1],
            _ptr(hyperplanes), s_t, w, t_ctx, block_pos0, q_pos0, 1 if causal else 0,
            n_anchor, n_local, k_exact, k_lsh, _ptr(keep_idx),
            _ptr(dbg_s_exact), _ptr(dbg_sig_k), _ptr(dbg_sig_q), _ptr(dbg_count), self._stream(stream))
        self._check(rc)

    def laserkv_append(self, k_blk, v_blk, keep_idx, *, b_t, block_pos0, k_cache, v_cache, cache_pos,
                       cache_len, stream=None):
        d = self.cfg.head_dim
        ks, vs = _strides3(k_blk, d), _strides3(v_blk, d)
        assert k_cache.stride(2) == 1 and k_cache.stride(1) == d and v_cache.stride() == k_cache.stride()
        rc = self._lib.laserkv_append(
            self._ctx, _ptr(k_blk), ks[0], ks[1], _ptr(v_blk), vs[0], vs[1], _ptr(keep_idx), b_t, k_blk.shape[1],
            block_pos0, _ptr(k_cache), _ptr(v_cache), k_cache.stride(0), _ptr(cache_pos), cache_pos.stride(0),
            cache_len, k_cache.shape[1], self._stream(stream))
        self._check(rc)

    def laserkv_compress_block(self, q_win, k_blk, v_blk, k_ctx, hyperplanes, *, block_pos0, q_pos0=None, causal=True,
                               n_anchor, n_local, k_exact, k_lsh, keep_idx, k_cache, v_cache, cache_pos, cache_len,
                               stream=None):
        d = self.cfg.head_dim
        s_t, w = k_blk.shape[1], q_win.shape[1]
        t_ctx = 0 if k_ctx is None else k_ctx.shape[1]
        if q_pos0 is None:
            q_pos0 = LKV_WINDOW_AT_BLOCK_END
        qs, ks, vs = _strides3(q_win, d), _strides3(k_blk, d), _strides3(v_blk, d)
        cs = _strides3(k_ctx, d) if k_ctx is not None else (0, 0)
        assert hyperplanes.is_contiguous()
        assert k_cache.stride(2) == 1 and k_cache.stride(1) == d and v_cache.stride() == k_cache.stride()
        rc = self._lib.laserkv_compress_block(
            self._ctx, _ptr(q_win), qs[0], qs[1], _ptr(k_blk), ks[0], ks[1], _ptr(v_blk), vs[0], vs[1],
            _ptr(k_ctx), cs[0], cs[1], _ptr(hyperplanes), s_t, w, t_ctx, block_pos0, q_pos0, 1 if causal else 0,
            n_anchor, n_local, k_exact, k_lsh, _ptr(keep_idx), _ptr(k_cache), _ptr(v_cache), k_cache.stride(0),
            _ptr(cache_pos), cache_pos.stride(0), cache_len, k_cache.shape[1], self._stream(stream))
        self._check(rc)

    def laserkv_score_block(self, q_win, k_blk, k_ctx, hyperplanes, *, block_pos0, q_pos0=None, causal=True,
                            score_acc, count_acc, accumulate, stream=None):
        d = self.cfg.head_dim
        s_t, w = k_blk.shape[1], q_win.shape[1]
        t_ctx = 0 if k_ctx is None else k_ctx.shape[1]
        if q_pos0 is None:
            q_pos0 = LKV_WINDOW_AT_BLOCK_END
        qs, ks = _strides3(q_win, d), _strides3(k_blk, d)
        cs = _strides3(k_ctx, d) if k_ctx is not None else (0, 0)
        assert hyperplanes.is_contiguous() and score_acc.is_contiguous() and count_acc.is_contiguous()
        assert score_acc.numel() >= s_t and count_acc.numel() >= s_t
        rc = self._lib.laserkv_score_block(
            self._ctx, _ptr(q_win), qs[0], qs[1], _ptr(k_blk), ks[0], ks[1], _ptr(k_ctx), cs[0], cs[1],
            _ptr(hyperplanes), s_t, w, t_ctx, block_pos0, q_pos0, 1 if causal else 0,
            _ptr(score_acc), _ptr(count_acc), 1 if accumulate else 0, self._stream(stream))
        self._check(rc)

    def laserkv_select_consensus(self, score_acc, count_acc, *, s_t, n_anchor, n_local, k_exact, k_lsh, keep_idx,
                                 stream=None):
        assert score_acc.is_contiguous() and count_acc.is_contiguous() and keep_idx.is_contiguous()
        rc = self._lib.laserkv_select_consensus(self._ctx, _ptr(score_acc), _ptr(count_acc), s_t, n_anchor, n_local,
                                                k_exact, k_lsh, _ptr(keep_idx), self._stream(stream))
        self._check(rc)

    def laserkv_append_shared(self, k_blk, v_blk, keep_idx, *, b_t, block_pos0, k_cache, v_cache, cache_pos,
                              cache_len, stream=None):
        d = self.cfg.head_dim
        ks, vs = _strides3(k_blk, d), _strides3(v_blk, d)
        assert k_cache.stride(2) == 1 and k_cache.stride(1) == d and v_cache.stride() == k_cache.stride()
        rc = self._lib.laserkv_append_shared(
            self._ctx, _ptr(k_blk), ks[0], ks[1], _ptr(v_blk), vs[0], vs[1], _ptr(keep_idx), b_t, k_blk.shape[1],
            block_pos0, _ptr(k_cache), _ptr(v_cache), k_cache.stride(0), _ptr(cache_pos), cache_pos.stride(0),
            cache_len, k_cache.shape[1], self._stream(stream))
        self._check(rc)

    def laserkv_set_row_lse(self, row_lse):
        """row_lse: contiguous float32 [H_q, w] device tensor, or None to switch the feature off.  The tensor
        is kept alive by this object for as long as it is set."""
        if row_lse is not None:
            assert row_lse.is_contiguous() and row_lse.dtype == self._torch.float32
        self._row_lse = row_lse
        self._check(self._lib.laserkv_set_row_lse(self._ctx, _ptr(row_lse)))

    def laserkv_set_row_lse_complete(self, row_lse):
        """row_lse: contiguous float32 [H_q, w] device tensor holding every window row's complete log-sum-exp,
        or None to let the library compute the statistics itself again."""
        if row_lse is not None:
            assert row_lse.is_contiguous() and row_lse.dtype == self._torch.float32
        self._row_lse = row_lse
        self._check(self._lib.laserkv_set_row_lse_complete(self._ctx, _ptr(row_lse)))

    def laserkv_attend_workspace_bytes(self, n_q, cache_len):
        n = int(self._lib.laserkv_attend_workspace_bytes(self._ctx, n_q, cache_len))
        if n < 0:
            raise LaserKVError(LKV_EINVAL, "attend_workspace_bytes: n_q or cache_len out of range")
        return n

    def laserkv_attend_cache(self, q, k_cache, v_cache, *, cache_len, out, out_lse, workspace, stream=None):
        """q [H_q, n_q, d]; k_cache / v_cache [H_kv, cap, d]; out float32 [H_q, n_q, d] or None (normaliser only),
        out_lse float32 [H_q, n_q];
        workspace: uint8 device tensor of at least laserkv_attend_workspace_bytes(n_q, cache_len) bytes."""
        d = self.cfg.head_dim
        qs = _strides3(q, d)
        assert k_cache.stride(2) == 1 and k_cache.stride(1) == d and v_cache.stride() == k_cache.stride()
        f32 = self._torch.float32
        assert out is None or (out.is_contiguous() and out.dtype == f32 and out.shape == q.shape)
        assert out_lse.is_contiguous() and out_lse.dtype == f32 and out_lse.shape == q.shape[:2]
        assert workspace.is_contiguous() and workspace.element_size() == 1
        rc = self._lib.laserkv_attend_cache(
            self._ctx, _ptr(q), qs[0], qs[1], q.shape[1], _ptr(k_cache), _ptr(v_cache), k_cache.stride(0), cache_len,
            _ptr(out), _ptr(out_lse), _ptr(workspace), workspace.numel(), self._stream(stream))
        self._check(rc)

    def laserkv_attend_block_workspace_bytes(self, n_q, cache_len, s_t):
        n = int(self._lib.laserkv_attend_block_workspace_bytes(self._ctx, n_q, cache_len, s_t))
        if n < 0:
            raise LaserKVError(LKV_EINVAL, "attend_block_workspace_bytes: n_q, cache_len or s_t out of range")
        return n

    def laserkv_attend_block(self, q, k_cache, v_cache, k_blk, v_blk, *, cache_len, block_pos0, q_pos0=None, causal=True,
                             out, out_lse, workspace, stream=None):
        """q [H_q, n_q, d]; k_cache / v_cache [H_kv, cap, d] (may be None with cache_len 0); k_blk / v_blk
        [H_kv, s_t, d] (views with strides allowed); out float32 [H_q, n_q, d], out_lse float32 [H_q, n_q];
        q_pos0 defaults to the block's last n_q positions;
        workspace: uint8 device tensor of at least laserkv_attend_block_workspace_bytes(n_q, cache_len, s_t) bytes."""
        d = self.cfg.head_dim
        qs, ks, vs = _strides3(q, d), _strides3(k_blk, d), _strides3(v_blk, d)
        s_t = k_blk.shape[1]
        assert v_blk.shape == k_blk.shape
        if k_cache is not None:
            assert k_cache.stride(2) == 1 and k_cache.stride(1) == d and v_cache.stride() == k_cache.stride()
        f32 = self._torch.float32
        assert out.is_contiguous() and out.dtype == f32 and out.shape == q.shape
        assert out_lse.is_contiguous() and out_lse.dtype == f32 and out_lse.shape == q.shape[:2]
        assert workspace.is_contiguous() and workspace.element_size() == 1
        if q_pos0 is None:
            q_pos0 = block_pos0 + s_t - q.shape[1]
        rc = self._lib.laserkv_attend_block(
            self._ctx, _ptr(q), qs[0], qs[1], q.shape[1], _ptr(k_cache), _ptr(v_cache),
            k_cache.stride(0) if k_cache is not None else 0, cache_len,
            _ptr(k_blk), ks[0], ks[1], _ptr(v_blk), vs[0], vs[1], s_t, block_pos0, q_pos0, 1 if causal else 0,
            _ptr(out), _ptr(out_lse), _ptr(workspace), workspace.numel(), self._stream(stream))
        self._check(rc)

    def laserkv_profile_begin(self):
        self._check(self._lib.laserkv_profile_begin(self._ctx))

    def laserkv_profile_end(self):
        """Returns {kernel name: (total ms, launches)}."""
        n = len(KERNEL_NAMES)
        ms = (C.c_double * n)()
        cnt = (C.c_int64 * n)()
        self._check(self._lib.laserkv_profile_end(self._ctx, ms, cnt))
        return {KERNEL_NAMES[i]: (float(ms[i]), int(cnt[i])) for i in range(n)}

    def laserkv_profile_isolate(self, kernel):
        """kernel: a name from KERNEL_NAMES, or None to launch every kernel again."""
        self._check(self._lib.laserkv_profile_isolate(self._ctx, -1 if kernel is None else KERNEL_NAMES.index(kernel)))
