"""Helpers shared by the GPU parity tests: move seeded inputs to the device, run
the HIP path through the binding, bring results back as numpy, compare."""
from __future__ import annotations

from typing import Dict

import numpy as np
import torch

from paper_2604_00785_amd import binding as B
from paper_2604_00785_amd import workloads as W

REL_TOL = 2e-2        # max |gpu - ref| / max |ref| per tensor: bf16 inputs, fp32 accumulation
GATE_TOL = 1e-5       # relative, fp32 softmax against the fp64 oracle


def bf16_to_dev(bits: np.ndarray, device="cuda:0") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).to(device).view(torch.bfloat16)


def bf16_from_dev(t: torch.Tensor) -> np.ndarray:
    """Device bf16 tensor -> float64 numpy (exact widening)."""
    bits = t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return W.bf16_bits_to_f32(bits).astype(np.float64)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    return W.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


class DeviceResults:
    """Results left on the device; rows are brought to the host on demand (large configs)."""

    def __init__(self, tensors: Dict[str, torch.Tensor]):
        self.t = tensors

    def _sel(self, name, idx):
        t = self.t[name]
        if idx is None:
            return t
        if isinstance(idx, slice):
            return t[idx]
        return t[torch.from_numpy(np.asarray(idx, dtype=np.int64)).to(t.device)]

    def rows(self, name, idx=None) -> np.ndarray:
        t = self._sel(name, idx)
        return bf16_from_dev(t) if t.dtype == torch.bfloat16 else t.cpu().numpy()

    def bits(self, name, idx=None) -> np.ndarray:
        return self._sel(name, idx).contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def run_layer(cfg: W.MoEConfig, inp: Dict[str, np.ndarray], device="cuda:0", keep_on_device=False, gather=False,
              fold=False):
    """Whole hot path on the GPU for one generated batch; returns numpy results
    (or a DeviceResults when keep_on_device is set).  gather: no xp, the GEMMs read x through row_token.
    fold: the gate weights are folded into h (results hw, ypw and row_weight instead of h, yp and dyp)."""
    buf = B.MoELayerBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, cfg.e_begin, cfg.n_local, cfg.renormalize, device,
                            gather=gather, fold=fold)
    x, dout = bf16_to_dev(inp["x"], device), bf16_to_dev(inp["dout"], device)
    Wg, Wu, Wd = (bf16_to_dev(inp[n], device) for n in ("Wg", "Wu", "Wd"))
    logits = torch.from_numpy(inp["logits"]).to(device)
    # poison outputs so that an element nobody wrote shows up
    for n in ("xp", "yp", "g", "u", "h", "dyp", "dxp", "out", "dx", "dWg", "dWu", "dWd"):
        if getattr(buf, n) is not None:
            getattr(buf, n).fill_(float("nan"))
    buf.run_fwd_bwd(x, logits, dout, Wg, Wu, Wd)
    torch.cuda.synchronize()
    if keep_on_device:
        return DeviceResults(buf.results())
    res = {}
    for n, t in buf.results().items():
        res[n] = bf16_from_dev(t) if t.dtype == torch.bfloat16 else t.cpu().numpy()
    return res


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    scale = np.abs(ref).max()
    if scale == 0.0:
        return float(np.abs(got).max())
    return float(np.abs(got - ref).max() / scale)


# Absolute floor of the element-wise check, in units of rms(ref).  Measured on the full-size workloads
# (printed by test_full_size_config): the 99.9th percentile of |d| / rms(ref) lies between 0.7e-2 (dgate)
# and 2.0e-2 (dxp), and weight gradients of experts with a handful of rows reach it too, so a floor below
# 2e-2 would flag more than the 1e-3 share of elements the check allows without any of them being wrong.
OUTLIER_FLOOR = 2e-2


def outlier_fraction(got: np.ndarray, ref: np.ndarray, floor: float = OUTLIER_FLOOR) -> float:
    """Share of elements off by more than 2e-2 relative plus `floor` * rms(ref).

    The floor covers elements near zero, whose error does not shrink with them: every result is a sum of
    products of values that were themselves rounded to bf16 (relative error up to 2^-9 = 2e-3 each), so an
    element's error is a few 1e-3 of the tensor's rms whatever its own size."""
    if ref.size == 0:
        return 0.0
    bad = np.abs(got - ref) > REL_TOL * np.abs(ref) + floor * ref_rms(ref)
    return float(bad.mean())


def ref_rms(ref: np.ndarray) -> float:
    return float(np.sqrt(np.mean(ref * ref))) if ref.size else 0.0


# (name, max|d|/max|ref|, p99.9 of |d|/rms(ref), max of |d|/rms(ref), outlier share) of every assert_close since the
# last clear: the full-size tests print it, so that the margins under the tolerances are on record.
ERR_LOG: list = []


def assert_close(got, ref, name, tol=REL_TOL):
    assert got.shape == ref.shape, (name, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), f"{name}: non-finite values (unwritten or overflowed elements)"
    e = rel_err(got, ref)
    fr = outlier_fraction(got, ref)
    rms = ref_rms(ref)
    if rms > 0.0:
        d = np.abs(got - ref).ravel() / rms
        ERR_LOG.append((name, e, float(np.quantile(d, 0.999)), float(d.max()), fr))
    assert e <= tol, f"{name}: max|d|/max|ref| = {e:.3e} > {tol}"
    assert fr <= 1e-3, f"{name}: {fr:.2e} of elements off by more than {REL_TOL} relative + {OUTLIER_FLOOR} rms"


def error_table() -> str:
    """ERR_LOG grouped by tensor (the part of the name in front of '['): worst case of each column."""
    worst: Dict[str, list] = {}
    for name, e, q, m, fr in ERR_LOG:
        key = name.split("[")[0]
        w = worst.setdefault(key, [0.0, 0.0, 0.0, 0.0, 0])
        w[0], w[1], w[2], w[3], w[4] = max(w[0], e), max(w[1], q), max(w[2], m), max(w[3], fr), w[4] + 1
    lines = ["%-8s %6s %16s %18s %14s %12s" % ("tensor", "checks", "max|d|/max|ref|", "p99.9 |d|/rms(ref)", "max |d|/rms", "outlier share")]
    for key, w in worst.items():
        lines.append("%-8s %6d %16.3e %18.3e %14.3e %12.2e" % (key, w[4], w[0], w[1], w[2], w[3]))
    return "\n".join(lines)


def row_weights(ref: Dict[str, np.ndarray]) -> np.ndarray:
    """Gate weight of every routed row of an oracle result: w_row[slot_row[t, i]] = topk_w[t, i]."""
    sr, w = ref["slot_row"], ref["topk_w"]
    out = np.zeros(int(ref["expert_offsets"][-1]), dtype=np.float64)
    out[sr[sr >= 0]] = w[sr >= 0]
    return out


def compare_layer(res: Dict[str, np.ndarray], ref: Dict[str, np.ndarray], n_local: int):
    """Bit-exact integer results, toleranced floating-point ones (rows < R only)."""
    for n in ("topk_idx", "expert_offsets", "slot_row"):
        assert np.array_equal(res[n], ref[n]), f"{n} differs"
    R = int(ref["expert_offsets"][-1])
    assert np.array_equal(res["row_token"][:R], ref["row_token"]), "row_token differs"
    np.testing.assert_allclose(res["topk_w"], ref["topk_w"], rtol=GATE_TOL, atol=1e-30)
    if "xp" in res:
        assert np.array_equal(res["xp"][:R], ref["xp"]), "xp is not an exact copy"
    if "hw" in res:      # gate weights folded into h: the oracle's h and yp times the row's weight; no dyp
        wr = row_weights(ref)
        np.testing.assert_allclose(res["row_weight"][:R], wr, rtol=GATE_TOL, atol=1e-30)
        assert_close(res["hw"][:R], ref["h"] * wr[:, None], "hw")
        assert_close(res["ypw"][:R], ref["yp"] * wr[:, None], "ypw")
        assert "dyp" not in res
        for n in ("g", "u", "dxp"):
            assert_close(res[n][:R], ref[n], n)
    else:
        for n in ("g", "u", "h", "yp", "dyp", "dxp"):
            assert_close(res[n][:R], ref[n], n)
    for n in ("out", "dx", "dgate"):
        assert_close(res[n], ref[n], n)
    off = ref["expert_offsets"]
    for n in ("dWg", "dWu", "dWd"):
        for e in range(n_local):
            if off[e] == off[e + 1]:
                assert np.all(res[n][e] == 0.0), f"{n}[{e}]: expert without rows must get zeros"
            else:
                assert_close(res[n][e], ref[n][e], f"{n}[{e}]")
