"""Seeded synthetic workloads shaped like the paper's long-context runs.

The paper evaluates on 16k / 64k / 128k-token contexts cut into 4k-class blocks
(Sec. 4; App. B) in which a few relevant facts sit in long filler (App. A).
That dataset is not available here, so these generators stand in for it: long
i.i.d. Gaussian filler with a few planted "needle" keys that align with the
block's window queries, plus the per-workload structure listed below.

This module holds input generation only: no scoring, hashing or selection
arithmetic.  It serves both the CPU oracle's tests and the HIP path so that both
see bit-identical storage-precision inputs.  The one quantity of the method it
needs, the number of protected positions at each block edge (needles are only
planted at selectable positions), is passed in by the caller.

Draw order per layer (one CPU torch.Generator, seed = BASE_SEED + 1000*c + layer):
hyperplanes, outlier channel indices, then per block: Q_win, K_blk, V_blk,
needle draws, per-key scale draws, duplicate draws.  Everything is produced in
fp32, modified, then rounded once to the storage dtype.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import torch

BASE_SEED = 260202199


@dataclass(frozen=True)
class Workload:
    name: str
    index: int              # position in the benchmark's list of configurations
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dtype: str              # "f32" | "bf16"
    l_ctx: int
    s_block: int
    window: int
    n_div: int              # protection divisor n
    lsh_tables: int         # L
    lsh_bits: int           # K
    n_layers: int = 1
    outlier_channels: int = 0
    outlier_scale: float = 8.0
    lognormal_sigma: float = 0.0
    needles_per_block: int = 0
    dup_fraction: float = 0.0
    r_num: int = 1          # compression ratio r = r_num / r_den (App. B: 0.25)
    r_den: int = 4
    alpha: float = 0.75     # exact share (Sec. 4.2)

    @property
    def n_blocks(self) -> int:
        return (self.l_ctx + self.s_block - 1) // self.s_block

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def torch_dtype(self):
        return torch.float32 if self.dtype == "f32" else torch.bfloat16


WORKLOADS = {
    "tiny": Workload("tiny", 0, 4, 2, 64, "f32", 4096, 512, 32, 4, 8, 8,
                     needles_per_block=2),
    "llama8b-16k": Workload("llama8b-16k", 1, 32, 8, 128, "bf16", 16384, 2048, 64, 4, 16, 10,
                            outlier_channels=4, needles_per_block=8),
    "llama8b-64k": Workload("llama8b-64k", 2, 32, 8, 128, "bf16", 65536, 2048, 64, 8, 16, 10,
                            n_layers=32, outlier_channels=4, needles_per_block=2),
    "llama8b-128k": Workload("llama8b-128k", 3, 32, 8, 128, "bf16", 131072, 4096, 128, 8, 32, 12,
                             outlier_channels=4, lognormal_sigma=0.5, needles_per_block=8),
    "gqa8-128k": Workload("gqa8-128k", 4, 64, 8, 128, "bf16", 131072, 8192, 64, 16, 32, 16,
                          outlier_channels=4, needles_per_block=8, dup_fraction=0.05),
}


def shrink(wl: Workload, **kw) -> Workload:
    """A smaller or altered copy of a workload (tests use it for ragged shapes)."""
    return replace(wl, **kw)


def _unit(x):
    return x / x.norm(dim=-1, keepdim=True).clamp_min(1e-30)


def _redirect(old, target_dir, cos):
    """Vector with old's norm whose cosine to target_dir is `cos`; the rest of its
    direction is old's component orthogonal to target_dir."""
    t = _unit(target_dir)
    perp = old - (old * t).sum(-1, keepdim=True) * t
    u = _unit(perp)
    new_dir = cos * t + (1.0 - cos * cos) ** 0.5 * u
    return new_dir * old.norm(dim=-1, keepdim=True)


def make_planes(wl: Workload, gen: torch.Generator):
    return torch.randn(wl.lsh_tables * wl.lsh_bits, wl.head_dim, generator=gen, dtype=torch.float32)


def make_layer(wl: Workload, layer: int = 0, n_protect: int = 0, n_blocks: int | None = None):
    """Generate one layer's inputs on the CPU.

    n_protect: positions at each block edge that are never selectable (needles
    and duplicates are planted strictly inside).
    n_blocks: generate only the first n_blocks blocks (same values as the full run).

    Returns a dict of CPU tensors in the storage dtype:
      planes [L*K, d], q_win [n_blocks, H_q, W, d], k [H_kv, n_blocks*S, d], v likewise,
      needles: int64 [n_needles, 3] rows (block, kv_head, block-local position).
    """
    gen = torch.Generator(device="cpu")
    gen.manual_seed(BASE_SEED + 1000 * wl.index + layer)
    nb = wl.n_blocks if n_blocks is None else min(n_blocks, wl.n_blocks)
    hq, hkv, d, s, w, g = wl.n_q_heads, wl.n_kv_heads, wl.head_dim, wl.s_block, wl.window, wl.group
    planes = make_planes(wl, gen)
    out_ch = None
    if wl.outlier_channels:
        out_ch = torch.randperm(d, generator=gen)[: wl.outlier_channels]
    lo, hi = n_protect, s - n_protect
    qs, ks, vs, needles = [], [], [], []
    for b in range(nb):
        s_t = min(s, wl.l_ctx - b * s)
        q = torch.randn(hq, w, d, generator=gen, dtype=torch.float32)
        k = torch.randn(hkv, s_t, d, generator=gen, dtype=torch.float32)
        v = torch.randn(hkv, s_t, d, generator=gen, dtype=torch.float32)
        if out_ch is not None:
            k[:, :, out_ch] *= wl.outlier_scale
        hi_t = min(hi, s_t - n_protect)
        if wl.needles_per_block and hi_t > lo:
            for h in range(hkv):
                pos = lo + torch.randperm(hi_t - lo, generator=gen)[: wl.needles_per_block]
                gi = torch.randint(0, g, (pos.numel(),), generator=gen)
                ji = torch.randint(0, w, (pos.numel(),), generator=gen)
                tgt = q[h * g + gi, ji]                       # [n, d]
                k[h, pos] = _redirect(k[h, pos], tgt, 0.9)
                for p in pos.tolist():
                    needles.append((b, h, p))
        if wl.lognormal_sigma:
            z = torch.randn(hkv, s_t, 1, generator=gen, dtype=torch.float32)
            k *= torch.exp(wl.lognormal_sigma * z)
        if wl.dup_fraction and hi_t > lo + 1:
            n_dup = int(wl.dup_fraction * (hi_t - lo))
            src_block = k.clone()
            for h in range(hkv):
                dst = lo + 1 + torch.randperm(hi_t - lo - 1, generator=gen)[:n_dup]
                u = torch.rand(n_dup, generator=gen)
                src = (u * dst.to(torch.float32)).floor().to(torch.int64).clamp_(0, s_t - 1)
                src = torch.minimum(src, dst - 1)
                exact = torch.arange(n_dup) < n_dup // 2
                copies = src_block[h, src]
                rnd = _unit(torch.randn(n_dup, d, generator=gen)) * copies.norm(dim=-1, keepdim=True)
                near = _redirect(rnd, copies, 0.99)
                k[h, dst] = torch.where(exact[:, None], copies, near)
        qs.append(q.to(wl.torch_dtype))
        ks.append(k.to(wl.torch_dtype))
        vs.append(v.to(wl.torch_dtype))
    return dict(
        planes=planes.to(wl.torch_dtype).contiguous(),
        q_win=torch.stack(qs).contiguous(),
        k=torch.cat(ks, dim=1).contiguous(),
        v=torch.cat(vs, dim=1).contiguous(),
        needles=torch.tensor(needles, dtype=torch.int64).reshape(-1, 3),
    )
