"""Thin ctypes binding over ``libmoe_hotpath.so`` (see ``include/moe_hotpath.h``).

Argument marshalling only: every step of the path runs in the HIP kernels.
torch tensors are used as device memory and for the current HIP stream.  There
is no CPU fallback: if the library is missing or a call fails, an exception is
raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Dict, List, Optional, Tuple

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libmoe_hotpath.so")

EXPORTS = [
    "moe_version", "moe_permute_workspace_bytes", "moe_grouped_gemm_bwd_workspace_bytes", "moe_workspace_bytes",
    "moe_route", "moe_permute", "moe_permute_bwd", "moe_grouped_gemm_fwd", "moe_grouped_gemm_bwd",
    "moe_grouped_gemm_fwd_gather", "moe_grouped_gemm_bwd_gather",
    "moe_permute_gate", "moe_route_permute", "moe_grouped_gemm_fwd_folded", "moe_unpermute_sum",
    "moe_grouped_gemm_bwd_folded_workspace_bytes", "moe_grouped_gemm_bwd_folded",
    "moe_unpermute_combine", "moe_unpermute_combine_bwd", "moe_prof_enable", "moe_prof_count", "moe_prof_read", "moe_prof_mfma_ceiling", "moe_prof_stream_read",
    "moe_router_fwd", "moe_route_bwd", "moe_router_bwd_workspace_bytes", "moe_router_bwd",
    "moe_permute_static_ws_capacity", "moe_permute_static_ws",
]

_ERR = {-1: "MOE_ERR_INVALID (bad pointer, alignment or size)", -2: "MOE_ERR_WORKSPACE (workspace too small)",
        -3: "MOE_ERR_LAUNCH (HIP launch failed)"}

_lib: Optional[ctypes.CDLL] = None


class MoeError(RuntimeError):
    pass


def load(build_if_missing: bool = True) -> ctypes.CDLL:
    """Loads the built library; builds it first only if no library is there."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        if not build_if_missing:
            raise MoeError(f"{LIB_PATH} is not built (run python -m paper_2604_00785_amd.build)")
        from . import build as _build
        _build.build(verbose=False)
    lib = ctypes.CDLL(LIB_PATH)
    c_int, c_sz, vp = ctypes.c_int, ctypes.c_size_t, ctypes.c_void_p
    lib.moe_version.restype = ctypes.c_char_p
    lib.moe_version.argtypes = []
    lib.moe_permute_workspace_bytes.restype = c_sz
    lib.moe_permute_workspace_bytes.argtypes = [c_int] * 3
    lib.moe_grouped_gemm_bwd_workspace_bytes.restype = c_sz
    lib.moe_grouped_gemm_bwd_workspace_bytes.argtypes = [c_int] * 2
    lib.moe_workspace_bytes.restype = c_sz
    lib.moe_workspace_bytes.argtypes = [c_int] * 5
    lib.moe_grouped_gemm_bwd_folded_workspace_bytes.restype = c_sz
    lib.moe_grouped_gemm_bwd_folded_workspace_bytes.argtypes = [c_int] * 2
    lib.moe_router_bwd_workspace_bytes.restype = c_sz
    lib.moe_router_bwd_workspace_bytes.argtypes = [c_int] * 3
    lib.moe_permute_static_ws_capacity.restype = c_sz
    lib.moe_permute_static_ws_capacity.argtypes = []
    sigs = {
        "moe_route": [vp, c_int, c_int, c_int, c_int, vp, vp, vp],
        "moe_permute": [vp, vp, c_int, c_int, c_int, c_int, c_int, c_int, vp, vp, vp, vp, vp, c_sz, vp],
        "moe_permute_static_ws": [vp, vp, c_int, c_int, c_int, c_int, c_int, c_int, vp, vp, vp, vp, vp],
        "moe_permute_bwd": [vp, vp, c_int, c_int, c_int, vp, vp],
        "moe_grouped_gemm_fwd": [vp, vp, vp, vp, vp, c_int, c_int, c_int, c_int, vp, vp, vp, vp, vp],
        "moe_grouped_gemm_bwd": [vp] * 9 + [c_int] * 4 + [vp] * 4 + [vp, c_sz, vp],
        "moe_grouped_gemm_fwd_gather": [vp, c_int, vp, vp, vp, vp, vp, c_int, c_int, c_int, c_int, vp, vp, vp, vp, vp],
        "moe_grouped_gemm_bwd_gather": [vp, vp, c_int, vp] + [vp] * 7 + [c_int] * 4 + [vp] * 4 + [vp, c_sz, vp],
        "moe_permute_gate": [vp, vp, c_int, c_int, c_int, c_int, c_int, vp, vp, vp, vp, vp, c_sz, vp],
        "moe_route_permute": [vp, vp, c_int, c_int, c_int, c_int, c_int, c_int, c_int, vp, vp, vp, vp, vp, vp, vp, vp, c_sz, vp],
        "moe_grouped_gemm_fwd_folded": [vp, c_int, vp, vp, vp, vp, vp, vp, c_int, c_int, c_int, c_int, vp, vp, vp, vp, vp],
        "moe_unpermute_sum": [vp, vp, c_int, c_int, c_int, vp, vp],
        "moe_grouped_gemm_bwd_folded": [vp, vp, c_int, c_int, vp, vp, vp] + [vp] * 7 + [c_int] * 4 + [vp] * 5 + [vp, c_sz, vp],
        "moe_unpermute_combine": [vp, vp, vp, c_int, c_int, c_int, vp, vp],
        "moe_unpermute_combine_bwd": [vp, vp, vp, vp, c_int, c_int, c_int, vp, vp, vp],
        "moe_router_fwd": [vp, vp, c_int, c_int, c_int, vp, vp],
        "moe_route_bwd": [vp, vp, vp, c_int, c_int, c_int, c_int, vp, vp],
        "moe_router_bwd": [vp, vp, vp, c_int, c_int, c_int, vp, vp, vp, c_sz, vp],
        "moe_prof_enable": [c_int],
        "moe_prof_count": [],
        "moe_prof_read": [c_int, ctypes.c_char_p, c_int, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(c_int)],
        "moe_prof_stream_read": [vp, c_sz, vp, c_int, vp],
        "moe_prof_mfma_ceiling": [vp, vp, c_int, c_int, vp, ctypes.POINTER(ctypes.c_float),
                                  ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double), vp],
    }
    for name, args in sigs.items():
        fn = getattr(lib, name)
        fn.restype = c_int
        fn.argtypes = args
    _lib = lib
    return lib


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise MoeError(f"{what} failed: {_ERR.get(rc, rc)}")


def _p(t: Optional[torch.Tensor]):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise MoeError("tensors must be contiguous device tensors")
    return ctypes.c_void_p(t.data_ptr())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _want(t: torch.Tensor, dtype, shape=None, name="tensor"):
    if t.dtype != dtype:
        raise MoeError(f"{name}: expected {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise MoeError(f"{name}: expected shape {tuple(shape)}, got {tuple(t.shape)}")


BF16 = torch.bfloat16


def moe_version() -> str:
    return load().moe_version().decode()


def moe_workspace_bytes(T: int, E: int, k: int, d: int, f: int) -> int:
    return int(load().moe_workspace_bytes(T, E, k, d, f))


def moe_permute_workspace_bytes(T: int, k: int, e_count: int) -> int:
    return int(load().moe_permute_workspace_bytes(T, k, e_count))


def moe_grouped_gemm_bwd_workspace_bytes(R_cap: int, f: int) -> int:
    return int(load().moe_grouped_gemm_bwd_workspace_bytes(R_cap, f))


def moe_route(logits, k: int, renormalize: int, topk_idx, topk_w) -> None:
    T, E = logits.shape
    _want(logits, torch.float32, name="logits")
    _want(topk_idx, torch.int32, (T, k), "topk_idx")
    _want(topk_w, torch.float32, (T, k), "topk_w")
    _check(load().moe_route(_p(logits), T, E, k, renormalize, _p(topk_idx), _p(topk_w), _stream()), "moe_route")


def moe_permute(x, topk_idx, E_total: int, e_begin: int, e_count: int,
                expert_offsets, row_token, slot_row, xp, ws) -> None:
    T, d = x.shape
    k = topk_idx.shape[1]
    _want(x, BF16, name="x")
    _want(topk_idx, torch.int32, (T, k), "topk_idx")
    _want(expert_offsets, torch.int32, (e_count + 1,), "expert_offsets")
    _want(row_token, torch.int32, (T * k,), "row_token")
    _want(slot_row, torch.int32, (T, k), "slot_row")
    if xp is not None:      # None: index arrays only (the *_gather products read x through row_token)
        _want(xp, BF16, (T * k, d), "xp")
    _check(load().moe_permute(_p(x), _p(topk_idx), T, d, E_total, k, e_begin, e_count, _p(expert_offsets),
                              _p(row_token), _p(slot_row), _p(xp), _p(ws), ws.numel() * ws.element_size(),
                              _stream()), "moe_permute")


def moe_permute_static_ws_capacity() -> int:
    return int(load().moe_permute_static_ws_capacity())


def moe_permute_static_ws(x, topk_idx, E_total: int, e_begin: int, e_count: int,
                          expert_offsets, row_token, slot_row, xp) -> None:
    """``moe_permute`` with the histogram table in the library's own device array (no workspace)."""
    T, d = x.shape
    k = topk_idx.shape[1]
    _want(x, BF16, name="x")
    _want(topk_idx, torch.int32, (T, k), "topk_idx")
    _want(expert_offsets, torch.int32, (e_count + 1,), "expert_offsets")
    _want(row_token, torch.int32, (T * k,), "row_token")
    _want(slot_row, torch.int32, (T, k), "slot_row")
    if xp is not None:
        _want(xp, BF16, (T * k, d), "xp")
    _check(load().moe_permute_static_ws(_p(x), _p(topk_idx), T, d, E_total, k, e_begin, e_count, _p(expert_offsets),
                                        _p(row_token), _p(slot_row), _p(xp), _stream()), "moe_permute_static_ws")


def moe_permute_bwd(dxp, slot_row, dx) -> None:
    T, k = slot_row.shape
    d = dxp.shape[1]
    _want(dxp, BF16, name="dxp")
    _want(slot_row, torch.int32, name="slot_row")
    _want(dx, BF16, (T, d), "dx")
    _check(load().moe_permute_bwd(_p(dxp), _p(slot_row), T, k, d, _p(dx), _stream()), "moe_permute_bwd")


def moe_grouped_gemm_fwd(xp, expert_offsets, Wg, Wu, Wd, g, u, h, yp) -> None:
    R_cap, d = xp.shape
    E, f, _ = Wg.shape
    for n, t, shp in (("xp", xp, (R_cap, d)), ("Wg", Wg, (E, f, d)), ("Wu", Wu, (E, f, d)), ("Wd", Wd, (E, d, f)),
                      ("g", g, (R_cap, f)), ("u", u, (R_cap, f)), ("h", h, (R_cap, f)), ("yp", yp, (R_cap, d))):
        _want(t, BF16, shp, n)
    _want(expert_offsets, torch.int32, (E + 1,), "expert_offsets")
    _check(load().moe_grouped_gemm_fwd(_p(xp), _p(expert_offsets), _p(Wg), _p(Wu), _p(Wd), E, R_cap, d, f,
                                       _p(g), _p(u), _p(h), _p(yp), _stream()), "moe_grouped_gemm_fwd")


def moe_grouped_gemm_fwd_gather(x, row_token, expert_offsets, Wg, Wu, Wd, g, u, h, yp) -> None:
    T, d = x.shape
    R_cap = row_token.shape[0]
    E, f, _ = Wg.shape
    for n, t, shp in (("x", x, (T, d)), ("Wg", Wg, (E, f, d)), ("Wu", Wu, (E, f, d)), ("Wd", Wd, (E, d, f)),
                      ("g", g, (R_cap, f)), ("u", u, (R_cap, f)), ("h", h, (R_cap, f)), ("yp", yp, (R_cap, d))):
        _want(t, BF16, shp, n)
    _want(row_token, torch.int32, (R_cap,), "row_token")
    _want(expert_offsets, torch.int32, (E + 1,), "expert_offsets")
    _check(load().moe_grouped_gemm_fwd_gather(_p(x), T, _p(row_token), _p(expert_offsets), _p(Wg), _p(Wu), _p(Wd), E,
                                              R_cap, d, f, _p(g), _p(u), _p(h), _p(yp), _stream()),
           "moe_grouped_gemm_fwd_gather")


def moe_grouped_gemm_bwd_gather(dyp, x, row_token, g, u, h, expert_offsets, Wg, Wu, Wd, dxp, dWg, dWu, dWd, ws) -> None:
    T, d = x.shape
    R_cap = row_token.shape[0]
    E, f, _ = Wg.shape
    for n, t, shp in (("dyp", dyp, (R_cap, d)), ("x", x, (T, d)), ("g", g, (R_cap, f)), ("u", u, (R_cap, f)),
                      ("h", h, (R_cap, f)), ("Wg", Wg, (E, f, d)), ("Wu", Wu, (E, f, d)), ("Wd", Wd, (E, d, f)),
                      ("dxp", dxp, (R_cap, d)), ("dWg", dWg, (E, f, d)), ("dWu", dWu, (E, f, d)),
                      ("dWd", dWd, (E, d, f))):
        _want(t, BF16, shp, n)
    _want(row_token, torch.int32, (R_cap,), "row_token")
    _want(expert_offsets, torch.int32, (E + 1,), "expert_offsets")
    _check(load().moe_grouped_gemm_bwd_gather(_p(dyp), _p(x), T, _p(row_token), _p(g), _p(u), _p(h),
                                              _p(expert_offsets), _p(Wg), _p(Wu), _p(Wd), E, R_cap, d, f, _p(dxp),
                                              _p(dWg), _p(dWu), _p(dWd), _p(ws), ws.numel() * ws.element_size(),
                                              _stream()), "moe_grouped_gemm_bwd_gather")


def moe_grouped_gemm_bwd(dyp, xp, g, u, h, expert_offsets, Wg, Wu, Wd, dxp, dWg, dWu, dWd, ws) -> None:
    R_cap, d = xp.shape
    E, f, _ = Wg.shape
    for n, t, shp in (("dyp", dyp, (R_cap, d)), ("xp", xp, (R_cap, d)), ("g", g, (R_cap, f)), ("u", u, (R_cap, f)),
                      ("h", h, (R_cap, f)), ("Wg", Wg, (E, f, d)), ("Wu", Wu, (E, f, d)), ("Wd", Wd, (E, d, f)),
                      ("dxp", dxp, (R_cap, d)), ("dWg", dWg, (E, f, d)), ("dWu", dWu, (E, f, d)),
                      ("dWd", dWd, (E, d, f))):
        _want(t, BF16, shp, n)
    _want(expert_offsets, torch.int32, (E + 1,), "expert_offsets")
    _check(load().moe_grouped_gemm_bwd(_p(dyp), _p(xp), _p(g), _p(u), _p(h), _p(expert_offsets), _p(Wg), _p(Wu),
                                       _p(Wd), E, R_cap, d, f, _p(dxp), _p(dWg), _p(dWu), _p(dWd), _p(ws),
                                       ws.numel() * ws.element_size(), _stream()), "moe_grouped_gemm_bwd")


def moe_grouped_gemm_bwd_folded_workspace_bytes(R_cap: int, f: int) -> int:
    return int(load().moe_grouped_gemm_bwd_folded_workspace_bytes(R_cap, f))


def moe_permute_gate(topk_idx, topk_w, E_total: int, e_begin: int, e_count: int,
                     expert_offsets, row_token, slot_row, row_weight, ws) -> None:
    T, k = topk_idx.shape
    _want(topk_idx, torch.int32, (T, k), "topk_idx")
    _want(topk_w, torch.float32, (T, k), "topk_w")
    _want(expert_offsets, torch.int32, (e_count + 1,), "expert_offsets")
    _want(row_token, torch.int32, (T * k,), "row_token")
    _want(slot_row, torch.int32, (T, k), "slot_row")
    _want(row_weight, torch.float32, (T * k,), "row_weight")
    _check(load().moe_permute_gate(_p(topk_idx), _p(topk_w), T, E_total, k, e_begin, e_count, _p(expert_offsets),
                                   _p(row_token), _p(slot_row), _p(row_weight), _p(ws),
                                   ws.numel() * ws.element_size(), _stream()), "moe_permute_gate")


def moe_route_permute(logits, x, k: int, renormalize: int, e_begin: int, e_count: int, topk_idx, topk_w,
                      expert_offsets, row_token, slot_row, row_weight, xp, ws) -> None:
    """Stages 1-3 in one call; ``x``/``xp`` and ``row_weight`` may be None."""
    T, E = logits.shape
    _want(logits, torch.float32, name="logits")
    _want(topk_idx, torch.int32, (T, k), "topk_idx")
    _want(topk_w, torch.float32, (T, k), "topk_w")
    _want(expert_offsets, torch.int32, (e_count + 1,), "expert_offsets")
    _want(row_token, torch.int32, (T * k,), "row_token")
    _want(slot_row, torch.int32, (T, k), "slot_row")
    d = 8
    if x is not None:
        _want(x, BF16, name="x")
        d = x.shape[1]
    if xp is not None:
        _want(xp, BF16, (T * k, d), "xp")
    if row_weight is not None:
        _want(row_weight, torch.float32, (T * k,), "row_weight")
    _check(load().moe_route_permute(_p(logits), _p(x), T, d, E, k, renormalize, e_begin, e_count, _p(topk_idx),
                                    _p(topk_w), _p(expert_offsets), _p(row_token), _p(slot_row), _p(row_weight),
                                    _p(xp), _p(ws), ws.numel() * ws.element_size(), _stream()), "moe_route_permute")


def moe_grouped_gemm_fwd_folded(x, row_token, row_weight, expert_offsets, Wg, Wu, Wd, g, u, hw, ypw) -> None:
    T, d = x.shape
    R_cap = row_token.shape[0]
    E, f, _ = Wg.shape
    for n, t, shp in (("x", x, (T, d)), ("Wg", Wg, (E, f, d)), ("Wu", Wu, (E, f, d)), ("Wd", Wd, (E, d, f)),
                      ("g", g, (R_cap, f)), ("u", u, (R_cap, f)), ("hw", hw, (R_cap, f)), ("ypw", ypw, (R_cap, d))):
        _want(t, BF16, shp, n)
    _want(row_token, torch.int32, (R_cap,), "row_token")
    _want(row_weight, torch.float32, (R_cap,), "row_weight")
    _want(expert_offsets, torch.int32, (E + 1,), "expert_offsets")
    _check(load().moe_grouped_gemm_fwd_folded(_p(x), T, _p(row_token), _p(row_weight), _p(expert_offsets), _p(Wg),
                                              _p(Wu), _p(Wd), E, R_cap, d, f, _p(g), _p(u), _p(hw), _p(ypw),
                                              _stream()), "moe_grouped_gemm_fwd_folded")


def moe_unpermute_sum(ypw, slot_row, out) -> None:
    T, k = slot_row.shape
    d = ypw.shape[1]
    _want(ypw, BF16, name="ypw")
    _want(slot_row, torch.int32, name="slot_row")
    _want(out, BF16, (T, d), "out")
    _check(load().moe_unpermute_sum(_p(ypw), _p(slot_row), T, k, d, _p(out), _stream()), "moe_unpermute_sum")


def moe_grouped_gemm_bwd_folded(dout, x, row_token, row_weight, slot_row, g, u, hw, expert_offsets, Wg, Wu, Wd,
                                dxp, dWg, dWu, dWd, dgate, ws) -> None:
    T, d = x.shape
    k = slot_row.shape[1]
    R_cap = row_token.shape[0]
    E, f, _ = Wg.shape
    for n, t, shp in (("dout", dout, (T, d)), ("x", x, (T, d)), ("g", g, (R_cap, f)), ("u", u, (R_cap, f)),
                      ("hw", hw, (R_cap, f)), ("Wg", Wg, (E, f, d)), ("Wu", Wu, (E, f, d)), ("Wd", Wd, (E, d, f)),
                      ("dxp", dxp, (R_cap, d)), ("dWg", dWg, (E, f, d)), ("dWu", dWu, (E, f, d)),
                      ("dWd", dWd, (E, d, f))):
        _want(t, BF16, shp, n)
    _want(row_token, torch.int32, (R_cap,), "row_token")
    _want(row_weight, torch.float32, (R_cap,), "row_weight")
    _want(slot_row, torch.int32, (T, k), "slot_row")
    _want(dgate, torch.float32, (T, k), "dgate")
    _want(expert_offsets, torch.int32, (E + 1,), "expert_offsets")
    _check(load().moe_grouped_gemm_bwd_folded(_p(dout), _p(x), T, k, _p(row_token), _p(row_weight), _p(slot_row),
                                              _p(g), _p(u), _p(hw), _p(expert_offsets), _p(Wg), _p(Wu), _p(Wd), E,
                                              R_cap, d, f, _p(dxp), _p(dWg), _p(dWu), _p(dWd), _p(dgate), _p(ws),
                                              ws.numel() * ws.element_size(), _stream()),
           "moe_grouped_gemm_bwd_folded")


def moe_unpermute_combine(yp, slot_row, topk_w, out) -> None:
    T, k = slot_row.shape
    d = yp.shape[1]
    _want(yp, BF16, name="yp")
    _want(slot_row, torch.int32, name="slot_row")
    _want(topk_w, torch.float32, (T, k), "topk_w")
    _want(out, BF16, (T, d), "out")
    _check(load().moe_unpermute_combine(_p(yp), _p(slot_row), _p(topk_w), T, k, d, _p(out), _stream()),
           "moe_unpermute_combine")


def moe_unpermute_combine_bwd(dout, yp, slot_row, topk_w, dyp, dgate) -> None:
    T, k = slot_row.shape
    d = yp.shape[1]
    _want(dout, BF16, (T, d), "dout")
    _want(yp, BF16, name="yp")
    _want(dyp, BF16, tuple(yp.shape), "dyp")
    _want(slot_row, torch.int32, name="slot_row")
    _want(topk_w, torch.float32, (T, k), "topk_w")
    _want(dgate, torch.float32, (T, k), "dgate")
    _check(load().moe_unpermute_combine_bwd(_p(dout), _p(yp), _p(slot_row), _p(topk_w), T, k, d, _p(dyp), _p(dgate),
                                            _stream()), "moe_unpermute_combine_bwd")


def moe_router_bwd_workspace_bytes(T: int, d: int, E: int) -> int:
    return int(load().moe_router_bwd_workspace_bytes(T, d, E))


def moe_router_fwd(x, Wr, logits) -> None:
    T, d = x.shape
    E = Wr.shape[0]
    _want(x, BF16, name="x")
    _want(Wr, torch.float32, (E, d), "Wr")
    _want(logits, torch.float32, (T, E), "logits")
    _check(load().moe_router_fwd(_p(x), _p(Wr), T, d, E, _p(logits), _stream()), "moe_router_fwd")


def moe_route_bwd(logits, topk_idx, dgate, renormalize: int, dlogits) -> None:
    T, E = logits.shape
    k = topk_idx.shape[1]
    _want(logits, torch.float32, name="logits")
    _want(topk_idx, torch.int32, (T, k), "topk_idx")
    _want(dgate, torch.float32, (T, k), "dgate")
    _want(dlogits, torch.float32, (T, E), "dlogits")
    _check(load().moe_route_bwd(_p(logits), _p(topk_idx), _p(dgate), T, E, k, renormalize, _p(dlogits), _stream()),
           "moe_route_bwd")


def moe_router_bwd(x, Wr, dlogits, dx, dWr, ws) -> None:
    """dWr is overwritten; the router's share of the input gradient is ADDED to dx."""
    T, d = x.shape
    E = Wr.shape[0]
    _want(x, BF16, name="x")
    _want(Wr, torch.float32, (E, d), "Wr")
    _want(dlogits, torch.float32, (T, E), "dlogits")
    _want(dx, BF16, (T, d), "dx")
    _want(dWr, torch.float32, (E, d), "dWr")
    _check(load().moe_router_bwd(_p(x), _p(Wr), _p(dlogits), T, d, E, _p(dx), _p(dWr), _p(ws),
                                 ws.numel() * ws.element_size(), _stream()), "moe_router_bwd")


def moe_prof_enable(on: bool) -> None:
    _check(load().moe_prof_enable(1 if on else 0), "moe_prof_enable")


def moe_prof_read() -> List[Tuple[str, float, int]]:
    """[(kernel name, total ms, launches)] recorded since profiling was enabled (synchronises)."""
    lib = load()
    out = []
    for i in range(lib.moe_prof_count()):
        buf = ctypes.create_string_buffer(64)
        ms, n = ctypes.c_float(), ctypes.c_int()
        _check(lib.moe_prof_read(i, buf, 64, ctypes.byref(ms), ctypes.byref(n)), "moe_prof_read")
        out.append((buf.value.decode(), float(ms.value), int(n.value)))
    return out


def moe_prof_mfma_ceiling(a: torch.Tensor, b: torch.Tensor, iters: int) -> Tuple[float, float]:
    """(TFLOP/s, core clock in GHz) of a pure MFMA loop on the operand values in ``a`` [n*512, 32]
    and ``b`` [n*512, 16] (bf16; n workgroups)."""
    n = a.shape[0] // 512
    assert a.dtype == BF16 and b.dtype == BF16 and a.shape == (n * 512, 32) and b.shape == (n * 512, 16)
    assert a.is_contiguous() and b.is_contiguous()
    sink = torch.empty(n * 512, dtype=torch.float32, device=a.device)
    ms, flop, ghz = ctypes.c_float(), ctypes.c_double(), ctypes.c_double()
    _check(load().moe_prof_mfma_ceiling(_p(a), _p(b), n, iters, _p(sink), ctypes.byref(ms), ctypes.byref(flop),
                                        ctypes.byref(ghz), _stream()), "moe_prof_mfma_ceiling")
    return flop.value / (ms.value * 1e-3) / 1e12, ghz.value


def moe_prof_stream_read(src: torch.Tensor, sink: torch.Tensor, workgroups: int) -> None:
    """Enqueue the read-only probe over ``src``; ``sink`` int32 [workgroups * 256]."""
    _want(sink, torch.int32, (workgroups * 256,), "sink")
    _check(load().moe_prof_stream_read(_p(src), src.numel() * src.element_size(), _p(sink), workgroups, _stream()),
           "moe_prof_stream_read")


class MoELayerBuffers:
    """Device buffers for one layer shape, allocated once (torch is the allocator).

    ``run_fwd_bwd`` enqueues the whole hot path - route, permute, grouped GEMM
    forward, combine, combine backward, grouped GEMM backward, permute backward -
    on the current stream, with no host synchronisation in between.
    """

    def __init__(self, T: int, d: int, E: int, k: int, f: int, e_begin: int = 0, e_count: int = -1,
                 renormalize: int = 1, device="cuda:0", gather: bool = False, fold: bool = False):
        self.T, self.d, self.E, self.k, self.f = T, d, E, k, f
        # fold: the gate weights are folded into h (``h`` and ``yp`` then hold hw and ypw, there is no dyp and
        # no separate backward of the combine); rows are gathered by the products, as with ``gather``
        if fold and T * d * 2 > 0xFFFFFFFF:
            raise MoeError("fold=True needs x under 4 GiB (32-bit row offsets)")
        self.fold = fold
        gather = gather or fold
        # True: no xp; the gate/up product and two weight gradients read x through row_token
        # (32-bit row offsets: x must stay under 4 GiB, else xp is materialised after all)
        gather = gather and T * d * 2 <= 0xFFFFFFFF
        self.gather = gather
        self.e_begin = e_begin
        self.e_count = E if e_count < 0 else e_count
        self.renormalize = renormalize
        dev = torch.device(device)
        nl, R = self.e_count, T * k
        z = lambda *s, dt=BF16: torch.zeros(*s, dtype=dt, device=dev)
        self.topk_idx = z(T, k, dt=torch.int32)
        self.topk_w = z(T, k, dt=torch.float32)
        self.expert_offsets = z(nl + 1, dt=torch.int32)
        self.row_token = z(R, dt=torch.int32)
        self.slot_row = z(T, k, dt=torch.int32)
        self.xp = None if gather else z(R, d)
        self.yp, self.dyp, self.dxp = z(R, d), (None if fold else z(R, d)), z(R, d)
        self.row_weight = z(R, dt=torch.float32) if fold else None
        self.g, self.u, self.h = z(R, f), z(R, f), z(R, f)
        self.out, self.dx = z(T, d), z(T, d)
        self.dgate = z(T, k, dt=torch.float32)
        self.dWg, self.dWu, self.dWd = z(nl, f, d), z(nl, f, d), z(nl, d, f)
        # one workspace for every call of the layer (the router's backward included)
        self.ws = torch.zeros(max(moe_workspace_bytes(T, E, k, d, f), 256), dtype=torch.uint8, device=dev)

    def run_fwd(self, x, logits, Wg, Wu, Wd) -> None:
        if self.fold:
            self._x = x
            moe_route_permute(logits, None, self.k, self.renormalize, self.e_begin, self.e_count, self.topk_idx,
                              self.topk_w, self.expert_offsets, self.row_token, self.slot_row, self.row_weight, None,
                              self.ws)
            moe_grouped_gemm_fwd_folded(x, self.row_token, self.row_weight, self.expert_offsets, Wg, Wu, Wd, self.g,
                                        self.u, self.h, self.yp)
            moe_unpermute_sum(self.yp, self.slot_row, self.out)
            return
        moe_route_permute(logits, x, self.k, self.renormalize, self.e_begin, self.e_count, self.topk_idx, self.topk_w,
                          self.expert_offsets, self.row_token, self.slot_row, None, self.xp, self.ws)
        if self.gather:
            self._x = x          # the backward reads the layer input again
            moe_grouped_gemm_fwd_gather(x, self.row_token, self.expert_offsets, Wg, Wu, Wd, self.g, self.u, self.h,
                                        self.yp)
        else:
            moe_grouped_gemm_fwd(self.xp, self.expert_offsets, Wg, Wu, Wd, self.g, self.u, self.h, self.yp)
        moe_unpermute_combine(self.yp, self.slot_row, self.topk_w, self.out)

    def run_bwd(self, dout, Wg, Wu, Wd) -> None:
        if self.fold:
            moe_grouped_gemm_bwd_folded(dout, self._x, self.row_token, self.row_weight, self.slot_row, self.g, self.u,
                                        self.h, self.expert_offsets, Wg, Wu, Wd, self.dxp, self.dWg, self.dWu,
                                        self.dWd, self.dgate, self.ws)
            moe_permute_bwd(self.dxp, self.slot_row, self.dx)
            return
        moe_unpermute_combine_bwd(dout, self.yp, self.slot_row, self.topk_w, self.dyp, self.dgate)
        if self.gather:
            moe_grouped_gemm_bwd_gather(self.dyp, self._x, self.row_token, self.g, self.u, self.h, self.expert_offsets,
                                        Wg, Wu, Wd, self.dxp, self.dWg, self.dWu, self.dWd, self.ws)
        else:
            moe_grouped_gemm_bwd(self.dyp, self.xp, self.g, self.u, self.h, self.expert_offsets, Wg, Wu, Wd,
                                 self.dxp, self.dWg, self.dWu, self.dWd, self.ws)
        moe_permute_bwd(self.dxp, self.slot_row, self.dx)

    def run_fwd_bwd(self, x, logits, dout, Wg, Wu, Wd) -> None:
        self.run_fwd(x, logits, Wg, Wu, Wd)
        self.run_bwd(dout, Wg, Wu, Wd)

    def run_block_fwd_bwd(self, x, Wr, dout, Wg, Wu, Wd) -> None:
        """The layer as a drop-in block: the router's Linear layer in front (logits from ``x`` and
        ``Wr``), and behind the expert path the gradient of the gates pushed back to the logits, to
        ``dWr`` and into ``dx`` (which then holds the expert path's and the router's share).  The
        buffers ``logits``, ``dlogits`` and ``dWr`` are created on first use."""
        if getattr(self, "logits", None) is None:
            dev = x.device
            self.logits = torch.zeros(self.T, self.E, dtype=torch.float32, device=dev)
            self.dlogits = torch.zeros(self.T, self.E, dtype=torch.float32, device=dev)
            self.dWr = torch.zeros(self.E, self.d, dtype=torch.float32, device=dev)
        moe_router_fwd(x, Wr, self.logits)
        self.run_fwd_bwd(x, self.logits, dout, Wg, Wu, Wd)
        moe_route_bwd(self.logits, self.topk_idx, self.dgate, self.renormalize, self.dlogits)
        moe_router_bwd(x, Wr, self.dlogits, self.dx, self.dWr, self.ws)   # the layer's one workspace is free again here

    def capture_fwd_bwd(self, x, logits, dout, Wg, Wu, Wd) -> "torch.cuda.CUDAGraph":
        """Record ``run_fwd_bwd`` on these buffers and arguments into a HIP graph.

        The entry points only launch kernels (no allocation, no memset, no host
        synchronisation), so the whole step can be captured; ``replay()`` then
        runs it again with one submission instead of a dozen launches.  Profiling
        (``moe_prof_enable``) must be off while capturing.
        """
        self.run_fwd_bwd(x, logits, dout, Wg, Wu, Wd)   # loads every kernel before the capture
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.run_fwd_bwd(x, logits, dout, Wg, Wu, Wd)
        return graph

    def results(self) -> Dict[str, torch.Tensor]:
        names = ("topk_idx", "topk_w", "expert_offsets", "row_token", "slot_row", "xp", "g", "u", "h", "yp", "out",
                 "dyp", "dgate", "dxp", "dWg", "dWu", "dWd", "dx", "row_weight")
        res = {n: getattr(self, n) for n in names if getattr(self, n) is not None}
        if self.fold:      # these two carry the gate weight of their row
            res["hw"], res["ypw"] = res.pop("h"), res.pop("yp")
        return res
