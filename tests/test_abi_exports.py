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
    # null pointers are rejected on the host before any GPU work
    lib = B.load()
    assert lib.moe_route(None, 1, 1, 1, 1, None, None, None) == -1
    assert lib.moe_unpermute_combine(None, None, None, 4, 2, 64, None, None) == -1
