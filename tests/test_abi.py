"""The C-ABI library loads, exports every symbol the header declares, and its host-only helpers agree
with the oracle (no GPU compute here)."""
import ctypes
import os
import re

import pytest

from oracle import laserkv_oracle as O
from paper_2602_02199_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2602_02199_amd import build
        build.build(verbose=False)
    return binding.load()


def test_every_declared_symbol_is_exported(lib):
    inc = os.path.join(ROOT, "include")
    header = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    declared = set(re.findall(r"\b(laserkv_[a-z_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_budget_matches_oracle(lib):
    for s, l in [(4096, 16384), (4096, 65536), (4096, 131072), (2048, 16384), (8192, 131072), (512, 4096), (1000, 7777)]:
        for rn, rd in [(1, 4), (1, 2), (3, 10)]:
            assert binding.laserkv_budget(s, l, rn, rd) == O.budget(s, l, rn, rd)
    with pytest.raises(binding.LaserKVError):
        binding.laserkv_budget(0, 10)


def test_partition_matches_oracle_and_rejects_bad_arguments(lib):
    for B, n, alpha, s_t in [(227, 4, 0.75, 512), (1985, 8, 0.75, 4096), (3855, 16, 0.75, 8192), (300, 3, 0.5, 100),
                             (7, 2, 0.3, 512), (1985, 8, 0.0, 4096), (1985, 8, 1.0, 4096)]:
        assert binding.laserkv_partition(B, n, alpha, s_t) == O.partition(B, n, alpha, s_t)
    for args in [(100, 1, 0.75, 512), (100, 4, 1.5, 512), (-1, 4, 0.5, 512), (100, 4, 0.5, 0)]:
        with pytest.raises(binding.LaserKVError) as ei:
            binding.laserkv_partition(*args)
        assert ei.value.code == binding.LKV_EINVAL


def test_create_rejects_bad_configs_without_touching_a_gpu(lib):
    bad = [dict(n_q_heads=5, n_kv_heads=2), dict(head_dim=96), dict(dtype=7), dict(lsh_bits=17), dict(lsh_tables=64, lsh_bits=16),
           dict(max_block=0), dict(max_window=4096)]
    base = dict(n_q_heads=4, n_kv_heads=2, head_dim=64, dtype=0, lsh_tables=8, lsh_bits=8, max_block=512, max_window=32,
                max_ctx_keys=64)
    for over in bad:
        cfg = binding.Config(**{**base, **over})
        out = ctypes.c_void_p()
        assert lib.laserkv_create(ctypes.byref(cfg), ctypes.byref(out)) == binding.LKV_EINVAL
        assert not out.value and lib.laserkv_last_error(None)


def test_static_workspace_size_is_reported_without_a_gpu(lib):
    small = binding.Config(4, 2, 64, 0, 8, 8, 512, 32, 56)
    bench = binding.Config(32, 8, 128, 1, 32, 12, 4096, 128, 248)
    huge = binding.Config(64, 64, 128, 1, 32, 12, 16384, 16, 4096)
    assert 0 < binding.laserkv_static_workspace_bytes(small) < binding.laserkv_static_workspace_bytes(bench)
    assert binding.laserkv_static_workspace_bytes(bench) <= binding.LKV_STATIC_SCRATCH_BYTES
    assert binding.laserkv_static_workspace_bytes(huge) > binding.LKV_STATIC_SCRATCH_BYTES
    assert binding.laserkv_static_workspace_bytes(binding.Config(5, 2, 64, 0, 8, 8, 512, 32, 56)) == 0
    header = open(os.path.join(ROOT, "include", "laserkv.h")).read()
    assert re.search(r"#define LKV_STATIC_SCRATCH_BYTES \(32u << 20\)", header) and binding.LKV_STATIC_SCRATCH_BYTES == 32 << 20


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/liblaserkv.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        binding.load()
