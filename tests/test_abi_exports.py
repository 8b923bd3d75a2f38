"""The C-ABI library loads without a GPU and exports every symbol the header declares."""
import ctypes
import os
import re

from paper_2604_00785_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_symbols():
    text = open(os.path.join(ROOT, "include", "moe_hotpath.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported_and_bound():
    lib = B.load()
    syms = header_symbols()
    assert len(syms) >= 14
    for s in syms:
        assert hasattr(lib, s), f"{s} declared in the header but not exported"
    assert set(syms) == set(B.EXPORTS)


def test_host_only_calls():
    assert "gfx950" in B.moe_version()
    assert B.moe_permute_workspace_bytes(8192, 8, 64) >= 64 * 64 * 4
    assert B.moe_grouped_gemm_bwd_workspace_bytes(65536, 1024) >= 2 * 65536 * 1024 * 2
    assert B.moe_workspace_bytes(8192, 64, 8, 2048, 1024) >= B.moe_grouped_gemm_bwd_workspace_bytes(65536, 1024)
    assert B.moe_workspace_bytes(0, 64, 8, 2048, 1024) == 0
    assert B.moe_workspace_bytes(1 << 30, 64, 8, 2048, 1024) == 0     # T*k does not fit an int
    # null pointers are rejected on the host before any GPU work
    lib = B.load()
    assert lib.moe_route(None, 1, 1, 1, 1, None, None, None) == -1
    assert lib.moe_unpermute_combine(None, None, None, 4, 2, 64, None, None) == -1


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    """No CPU fallback: without the built library the binding raises, and it refuses host tensors."""
    import pytest
    import torch
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", str(tmp_path / "libmoe_hotpath_absent.so"))
    with pytest.raises(B.MoeError):
        B.load(build_if_missing=False)
    monkeypatch.undo()
    logits = torch.zeros(4, 4)
    idx = torch.zeros(4, 2, dtype=torch.int32)
    w = torch.zeros(4, 2)
    with pytest.raises(B.MoeError):
        B.moe_route(logits, 2, 1, idx, w)


def test_host_only_calls_router_and_gather():
    lib = B.load()
    assert B.moe_router_bwd_workspace_bytes(8192, 2048, 64) == 32 * 64 * 2048 * 4   # one partial sum per 256 tokens
    assert B.moe_router_bwd_workspace_bytes(0, 2048, 64) == 0
    assert lib.moe_router_fwd(None, None, 64, 64, 8, None, None) == -1
    assert lib.moe_route_bwd(None, None, None, 64, 8, 2, 1, None, None) == -1
    assert lib.moe_router_bwd(None, None, None, 64, 64, 8, None, None, None, 0, None) == -1
    assert lib.moe_grouped_gemm_fwd_gather(None, 64, None, None, None, None, None, 1, 64, 64, 64,
                                           None, None, None, None, None) == -1
    assert lib.moe_grouped_gemm_bwd_gather(None, None, 64, None, None, None, None, None, None, None, None,
                                           1, 64, 64, 64, None, None, None, None, None, 0, None) == -1


def test_forced_uniform_routing_workload():
    """The forced-uniform-routing logits give every expert exactly T*k/E rows, slot i of token t on
    expert (t*k + i) mod E, in decreasing order of the logits."""
    import numpy as np
    from oracle import moe_oracle as O
    from paper_2604_00785_amd import workloads as W
    T, E, k = 96, 16, 4
    logits = W.fur_logits(T, E, k)
    idx, w = O.route(logits, k, 1)
    want = (np.arange(T)[:, None] * k + np.arange(k)[None, :]) % E
    assert np.array_equal(idx, want)
    assert np.all(np.bincount(idx.ravel(), minlength=E) == T * k // E)
    assert np.all(np.diff(w, axis=1) < 0)
    for name in ("mula100b_ep12", "mula220b_ep12", "olmoe_fur"):
        cfg = W.CONFIGS[name]
        assert cfg.e_begin + cfg.n_local <= cfg.E and cfg.d % 64 == 0 and cfg.f % 64 == 0


def test_host_only_calls_folded_gate_weights():
    lib = B.load()
    base = B.moe_grouped_gemm_bwd_workspace_bytes(65536, 1024)
    assert B.moe_grouped_gemm_bwd_folded_workspace_bytes(65536, 1024) == base + 16 * 65536 * 4   # one fp32 per row and 64-column strip
    assert B.moe_grouped_gemm_bwd_folded_workspace_bytes(0, 1024) == 0
    assert lib.moe_permute_gate(None, None, 64, 8, 2, 0, 8, None, None, None, None, None, 0, None) == -1
    assert lib.moe_unpermute_sum(None, None, 4, 2, 64, None, None) == -1
    assert lib.moe_grouped_gemm_fwd_folded(None, 64, None, None, None, None, None, None, 1, 64, 64, 64,
                                           None, None, None, None, None) == -1
    assert lib.moe_grouped_gemm_bwd_folded(None, None, 64, 2, None, None, None, None, None, None, None, None, None,
                                           None, 1, 64, 64, 64, None, None, None, None, None, None, 0, None) == -1


def test_moe_workspace_bytes_covers_every_call():
    """The one-size-fits-all bound is at least every specific workspace size, over a grid of shapes
    (among them one where the router's partial sums are the largest, and the headline shape, where
    the folded backward product's are)."""
    import itertools
    shapes = list(itertools.product((1, 256, 8192, 16384), (1, 8, 64, 512), (1, 2, 8), (64, 2048, 4096), (64, 512, 1024)))
    shapes += [(8192, 64, 1, 4096, 64), (8192, 64, 8, 2048, 1024), (32768, 64, 8, 4096, 2048)]
    for T, E, k, d, f in shapes:
        if k > E:
            continue
        total = B.moe_workspace_bytes(T, E, k, d, f)
        parts = {
            "permute": B.moe_permute_workspace_bytes(T, k, E),
            "bwd": B.moe_grouped_gemm_bwd_workspace_bytes(T * k, f),
            "bwd_folded": B.moe_grouped_gemm_bwd_folded_workspace_bytes(T * k, f),
            "router_bwd": B.moe_router_bwd_workspace_bytes(T, d, E),
        }
        for name, v in parts.items():
            assert total >= v, (name, (T, E, k, d, f), total, v)
        assert total == max(parts.values())
    assert B.moe_workspace_bytes(8192, 64, 8, 2048, 1024) == B.moe_grouped_gemm_bwd_folded_workspace_bytes(65536, 1024)
    assert B.moe_workspace_bytes(8192, 64, 1, 4096, 64) == B.moe_router_bwd_workspace_bytes(8192, 4096, 64)
