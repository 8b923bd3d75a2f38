"""moe_permute_static_ws (the entry point that takes no workspace and allocates nothing) against
moe_permute and the oracle, through the C ABI: two calls in a row, the second on a smaller input, so
that whatever the first call left in the library's device array is still there."""
import ctypes

import numpy as np
import pytest
import torch

import gpu_harness as H
from oracle import moe_oracle as O
from paper_2604_00785_amd import binding as B
from paper_2604_00785_amd import workloads as W

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _run_case(lib, T, E, k, d, eb, ec, seed, with_rows):
    print(f"static-ws permute T={T} E={E} k={k} d={d} local=[{eb},{eb + ec}) rows={with_rows}", flush=True)
    rng = np.random.default_rng(seed)
    idx = np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)
    xb = W.f32_to_bf16_bits(rng.standard_normal((T, d)).astype(np.float32))
    x = H.bf16_to_dev(xb)
    idx_d = torch.from_numpy(idx).to(DEV)
    R_cap = T * k
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

    def outputs():
        return (torch.full((ec + 1,), -7, dtype=torch.int32, device=DEV),
                torch.full((R_cap,), -7, dtype=torch.int32, device=DEV),
                torch.full((T, k), -7, dtype=torch.int32, device=DEV),
                torch.full((R_cap, d), float("nan"), dtype=torch.bfloat16, device=DEV) if with_rows else None)

    off_a, rt_a, sr_a, xp_a = outputs()     # existing entry point, caller's workspace
    ws = torch.zeros(max(B.moe_permute_workspace_bytes(T, k, ec), 16), dtype=torch.uint8, device=DEV)
    rc = lib.moe_permute(_ptr(x), _ptr(idx_d), T, d, E, k, eb, ec, _ptr(off_a), _ptr(rt_a), _ptr(sr_a), _ptr(xp_a),
                         _ptr(ws), ws.numel(), stream)
    assert rc == 0
    off_b, rt_b, sr_b, xp_b = outputs()     # the one that takes no workspace
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    rc = lib.moe_permute_static_ws(_ptr(x), _ptr(idx_d), T, d, E, k, eb, ec, _ptr(off_b), _ptr(rt_b), _ptr(sr_b),
                                   _ptr(xp_b), stream)
    assert rc == 0
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    # bit-exact against the existing entry point (integer work and a plain copy)
    assert torch.equal(off_a, off_b) and torch.equal(rt_a, rt_b) and torch.equal(sr_a, sr_b)
    if with_rows:
        R = int(off_a[-1])
        assert torch.equal(xp_a[:R].view(torch.int16), xp_b[:R].view(torch.int16))
        assert bool(torch.isnan(xp_b[R:]).all())          # rows past R untouched
    # and against the oracle
    roff, rrt, rsr, rxp = O.permute(O.decode_bf16(xb), idx, eb, ec)
    R = int(roff[-1])
    assert np.array_equal(off_b.cpu().numpy(), roff)
    assert np.array_equal(sr_b.cpu().numpy(), rsr)
    assert np.array_equal(rt_b.cpu().numpy()[:R], rrt)
    assert np.all(rt_b.cpu().numpy()[R:] == -7)
    if with_rows:
        assert np.array_equal(H.bf16_from_dev(xp_b)[:R], rxp)


def test_static_workspace_permute_matches_moe_permute_twice():
    lib = B.load(build_if_missing=False)
    cap = B.moe_permute_static_ws_capacity()
    assert cap == 1 << 20
    # first a table that fills a good part of the array (128 experts x 512 workgroups = 256 KiB), then
    # a much smaller one that reuses its first cells, then an expert-parallel share without row copies
    _run_case(lib, 16384, 128, 8, 64, 0, 128, seed=1, with_rows=True)
    _run_case(lib, 1000, 64, 8, 256, 0, 64, seed=2, with_rows=True)
    _run_case(lib, 777, 64, 8, 128, 16, 8, seed=3, with_rows=False)


def test_static_workspace_permute_refuses_what_does_not_fit():
    lib = B.load(build_if_missing=False)
    cap = B.moe_permute_static_ws_capacity()
    T, E, k, d = 70000, 512, 8, 8            # 512 experts x 2188 workgroups x 4 bytes > 1 MiB
    assert B.moe_permute_workspace_bytes(T, k, E) > cap
    x = torch.zeros(T, d, dtype=torch.bfloat16, device=DEV)
    idx = torch.zeros(T, k, dtype=torch.int32, device=DEV)
    off = torch.full((E + 1,), -7, dtype=torch.int32, device=DEV)
    rt = torch.full((T * k,), -7, dtype=torch.int32, device=DEV)
    sr = torch.full((T, k), -7, dtype=torch.int32, device=DEV)
    rc = lib.moe_permute_static_ws(_ptr(x), _ptr(idx), T, d, E, k, 0, E, _ptr(off), _ptr(rt), _ptr(sr), None, None)
    assert rc == -2                          # MOE_ERR_WORKSPACE, nothing enqueued
    torch.cuda.synchronize()
    assert bool((off == -7).all()) and bool((sr == -7).all())
    # invalid arguments are still refused as by moe_permute
    assert lib.moe_permute_static_ws(None, None, 16, 8, 4, 2, 0, 4, None, None, None, None, None) == -1
