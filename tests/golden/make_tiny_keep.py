#!/usr/bin/env python3
"""Writes tests/golden/tiny_keep_sets.txt: the oracle's kept index sets for the first two blocks of the
tiny workload (layer 0).  Calls only the oracle and the seeded input generator; the file guards the
oracle and the generator against silent drift (it is not an independent pin of either).

Run from the repository root:  python tests/golden/make_tiny_keep.py
"""
import hashlib
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import laserkv_oracle as O  # noqa: E402
from paper_2602_02199_amd import synth  # noqa: E402


def compute():
    wl = synth.WORKLOADS["tiny"]
    B = O.budget(wl.s_block, wl.l_ctx, wl.r_num, wl.r_den)
    parts = O.partition(B, wl.n_div, wl.alpha, wl.s_block)
    data = synth.make_layer(wl, 0, parts[0], n_blocks=2)
    k = data["k"].double().numpy()
    q = data["q_win"].double().numpy()
    planes = data["planes"].double().numpy()
    lines = []
    s = wl.s_block
    for t in range(2):
        k_ctx = k[:, t * s - parts[1]:t * s] if t else None
        st = O.select_block(q[t], k[:, t * s:(t + 1) * s], k_ctx, planes, wl.lsh_tables, wl.lsh_bits, *parts,
                            block_pos0=t * s)
        for h in range(wl.n_kv_heads):
            keep = st["keep"][h]
            digest = hashlib.sha256(np.asarray(keep, dtype=np.int64).tobytes()).hexdigest()[:16]
            lines.append(f"{t} {h} {len(keep)} {int(keep[60])} {int(keep[120])} {int(keep[-60])} "
                         f"{int(st['cnt'][h].sum())} {digest}")
    return lines


HEADER = ("# oracle kept sets, tiny workload, layer 0, blocks 0-1 (written by tests/golden/make_tiny_keep.py)\n"
          "# columns: block kv_head n_kept keep[60] keep[120] keep[-60] sum_of_counts sha256(keep as int64)[:16]\n")

if __name__ == "__main__":
    out = os.path.join(os.path.dirname(os.path.abspath(__file__)), "tiny_keep_sets.txt")
    with open(out, "w") as f:
        f.write(HEADER + "\n".join(compute()) + "\n")
    print(open(out).read())
