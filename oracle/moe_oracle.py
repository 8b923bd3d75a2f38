"""Plain, slow, obviously-correct CPU definition of the SparseMoE expert layer.

TEST INFRASTRUCTURE ONLY: imported by ``tests/``, ``__graft_entry__.smoke()``
and the ``cpu_baseline`` leg of ``bench.py``; never by the product path.  It
shares no code with the HIP kernels or their Python binding.

What is defined here (paper: Section 3.1 "FastSparseMoE" and Algorithm 1):

* ``route``            Stage 1: ``probs = Softmax(logits)``, ``weights, indices = TopK(probs)``.
* ``permute``          Stages 2-3 and the first line of Stage 4: per-expert token counts,
                       their prefix sum (``cum_token_counts``), ``input_indices`` /
                       ``output_indices`` and ``mlp_in = input[input_indices]``.
* ``expert_mlp_fwd``   Stage 4: three grouped matrix products around ``Silu(gate) * up``.
* ``combine_fwd``      Stage 5, ExpertOutputReductionForward.
* ``combine_bwd``      Stage 5, ExpertOutputReductionBackward.
* ``expert_mlp_bwd``   derivative of Stage 4 (the paper leaves it to autograd).
* ``permute_bwd``      derivative of the Stage-4 gather (likewise).
* ``router_logits``    Stage 1, ``logits = Router(input)`` (the router is a Linear layer without bias).
* ``route_bwd``        derivative of Stage 1's Softmax / TopK / renormalisation with respect to the
                       logits, for a given gradient of the k gate weights (autograd in the paper).
* ``router_bwd``       derivative of the router's Linear layer: its weight gradient and its share of
                       the gradient of the layer input.

The paper's method is a re-organisation of the dropless top-k SwiGLU MoE layer,
not an approximation of it, so every function is the plain definition written
out: the permutation is a stable sort of the (token, slot) pairs by expert id,
the grouped products are one matrix product per expert, and so on.  There is no
blocking, fusion or reordering.  All floating-point work is done in fp64 (pass
``dtype=np.float32`` for the fp32 variant); bfloat16 inputs arrive as uint16 bit
patterns and are widened exactly; nothing is rounded back to bfloat16.

Readings taken where the paper is silent (all listed again in the design notes):
top-k ties go to the lower expert id; slots are ordered by decreasing
probability; selection compares the logits (softmax is monotone, so this is
TopK(Softmax(logits)) in exact arithmetic); ``renormalize`` divides the k gates
by their sum (Algorithm 1 uses the TopK weights as they are: ``renormalize=0``);
no biases anywhere; ``n_end`` of Algorithm 1 is inclusive.

Pins: every function here is checked by ``tests/test_oracle_*.py`` against
brute force on tiny inputs, the per-token dense definition, library autograd,
finite differences and the invariants the paper's text fixes.  The paper prints
no numeric example for this path (its one worked example is a figure), so there
is no printed-value pin.
"""
from __future__ import annotations

from typing import Dict, Tuple

import numpy as np


def decode_bf16(bits: np.ndarray, dtype=np.float64) -> np.ndarray:
    """Widen bfloat16 bit patterns (uint16) exactly."""
    b = np.asarray(bits, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(dtype)


# --------------------------------------------------------------------------
# Stage 1 (Algorithm 1, the Softmax and TopK lines)
# --------------------------------------------------------------------------
def route(logits: np.ndarray, k: int, renormalize: int = 1,
          dtype=np.float64) -> Tuple[np.ndarray, np.ndarray]:
    """Softmax over experts, then the k largest per token.

    logits [T, E] fp32.  Returns ``topk_idx`` int32 [T, k] (slot i = i-th
    largest, equal logits -> lower expert id first) and ``topk_w`` [T, k], the
    softmax probabilities of the chosen experts, divided by their sum when
    ``renormalize`` is set.
    """
    logits = np.asarray(logits, dtype=np.float32)
    T, E = logits.shape
    assert 1 <= k <= E
    # a stable sort of the negated logits keeps equal values in expert order
    order = np.argsort(-logits, axis=1, kind="stable")
    topk_idx = order[:, :k].astype(np.int32)
    l = logits.astype(dtype)
    z = np.exp(l - l.max(axis=1, keepdims=True))
    probs = z / z.sum(axis=1, keepdims=True)
    topk_w = np.take_along_axis(probs, topk_idx.astype(np.int64), axis=1)
    if renormalize:
        topk_w = topk_w / topk_w.sum(axis=1, keepdims=True)
    return topk_idx, topk_w


def router_logits(x: np.ndarray, Wr: np.ndarray) -> np.ndarray:
    """Stage 1, first line: logits[t, e] = sum_j x[t, j] * Wr[e, j] (a Linear layer, no bias)."""
    return np.asarray(x) @ np.asarray(Wr, dtype=np.asarray(x).dtype).T


def route_bwd(logits: np.ndarray, topk_idx: np.ndarray, dgate: np.ndarray, renormalize: int = 1,
              dtype=np.float64) -> np.ndarray:
    """Gradient with respect to the logits, given dgate[t, i] = dL/d topk_w[t, i].

    The chosen experts are held fixed (TopK passes the gradient to the chosen
    entries and nothing to the others).  With p = Softmax(logits), s_i = p[idx_i]
    and S = sum_i s_i:  topk_w_i = s_i / S when renormalising, else s_i.
      renormalised:   dL/ds_i = (dgate_i - sum_j dgate_j * topk_w_j) / S
      otherwise:      dL/ds_i = dgate_i
    dL/dp_e = dL/ds_i where e = idx_i, else 0, and through the softmax
      dlogits_e = p_e * (dL/dp_e - sum_e' dL/dp_e' * p_e').
    """
    l = np.asarray(logits, dtype=np.float32).astype(dtype)
    idx = np.asarray(topk_idx).astype(np.int64)
    dgate = np.asarray(dgate, dtype=dtype)
    z = np.exp(l - l.max(axis=1, keepdims=True))
    p = z / z.sum(axis=1, keepdims=True)
    s = np.take_along_axis(p, idx, axis=1)
    if renormalize:
        S = s.sum(axis=1, keepdims=True)
        w = s / S
        ds = (dgate - (dgate * w).sum(axis=1, keepdims=True)) / S
    else:
        ds = dgate
    dp = np.zeros_like(p)
    np.put_along_axis(dp, idx, ds, axis=1)
    return p * (dp - (dp * p).sum(axis=1, keepdims=True))


def router_bwd(x: np.ndarray, Wr: np.ndarray, dlogits: np.ndarray):
    """Derivative of ``logits = x @ Wr.T``: dWr = dlogits.T @ x, dx = dlogits @ Wr."""
    x = np.asarray(x)
    Wr = np.asarray(Wr, dtype=x.dtype)
    dl = np.asarray(dlogits, dtype=x.dtype)
    return dl.T @ x, dl @ Wr


# --------------------------------------------------------------------------
# Stages 2-3 (token counting, index generation) and the Stage-4 gather
# --------------------------------------------------------------------------
def permute(x: np.ndarray, topk_idx: np.ndarray, e_begin: int, e_count: int):
    """Group the (token, slot) pairs by local expert, keeping token order.

    Returns
      expert_offsets int32 [e_count+1]  exclusive prefix sum of per-expert
                                        counts (Algorithm 1: cum_token_counts)
      row_token      int32 [R]          token of each grouped row (input_indices)
      slot_row       int32 [T, k]       grouped row of each pair, -1 when the
                                        expert is not local (dense form of
                                        output_indices / selected_expert_indices)
      xp             x.dtype [R, d]     x[row_token]  (mlp_in)
    """
    topk_idx = np.asarray(topk_idx)
    T, k = topk_idx.shape
    flat = topk_idx.reshape(-1).astype(np.int64)
    is_local = (flat >= e_begin) & (flat < e_begin + e_count)
    by_expert = np.argsort(flat, kind="stable")          # pair ids, expert-major, pair order kept
    by_expert = by_expert[is_local[by_expert]]
    counts = np.bincount(flat[is_local] - e_begin, minlength=e_count)
    expert_offsets = np.zeros(e_count + 1, dtype=np.int32)
    expert_offsets[1:] = np.cumsum(counts)
    R = int(expert_offsets[-1])
    row_token = (by_expert // k).astype(np.int32)
    slot_row = np.full(T * k, -1, dtype=np.int32)
    slot_row[by_expert] = np.arange(R, dtype=np.int32)
    xp = np.asarray(x)[row_token]
    return expert_offsets, row_token, slot_row.reshape(T, k), xp


def permute_bwd(dxp: np.ndarray, slot_row: np.ndarray) -> np.ndarray:
    """Derivative of ``xp = x[row_token]``: dx[t] = sum of dxp over t's rows."""
    T, k = slot_row.shape
    dx = np.zeros((T, dxp.shape[1]), dtype=dxp.dtype)
    for i in range(k):
        rows = slot_row[:, i]
        m = rows >= 0
        dx[m] += dxp[rows[m]]
    return dx


# --------------------------------------------------------------------------
# Stage 4 (expert computation) and its derivative
# --------------------------------------------------------------------------
def _sigmoid(z):
    return 1.0 / (1.0 + np.exp(-z))


def expert_mlp_fwd(xp, expert_offsets, Wg, Wu, Wd) -> Dict[str, np.ndarray]:
    """gate/up products, Silu(gate)*up, down product, one expert at a time.

    xp [R, d]; Wg, Wu [n_local, f, d]; Wd [n_local, d, f] (each expert's
    ``[out, in]`` weight, stacked).  Returns g, u, h [R, f] and yp [R, d].
    """
    R, d = xp.shape
    nl, f, _ = Wg.shape
    g = np.zeros((R, f), dtype=xp.dtype)
    u = np.zeros((R, f), dtype=xp.dtype)
    h = np.zeros((R, f), dtype=xp.dtype)
    yp = np.zeros((R, d), dtype=xp.dtype)
    for e in range(nl):
        a, b = int(expert_offsets[e]), int(expert_offsets[e + 1])
        if a == b:
            continue
        g[a:b] = xp[a:b] @ Wg[e].T
        u[a:b] = xp[a:b] @ Wu[e].T
        h[a:b] = g[a:b] * _sigmoid(g[a:b]) * u[a:b]
        yp[a:b] = h[a:b] @ Wd[e].T
    return {"g": g, "u": u, "h": h, "yp": yp}


def expert_mlp_bwd(dyp, xp, g, u, h, expert_offsets, Wg, Wu, Wd) -> Dict[str, np.ndarray]:
    """Chain rule through Stage 4.  Experts without rows get exactly zero dW."""
    R, d = xp.shape
    nl, f, _ = Wg.shape
    dxp = np.zeros_like(xp)
    dg = np.zeros_like(g)
    du = np.zeros_like(u)
    dWg = np.zeros_like(Wg)
    dWu = np.zeros_like(Wu)
    dWd = np.zeros_like(Wd)
    for e in range(nl):
        a, b = int(expert_offsets[e]), int(expert_offsets[e + 1])
        if a == b:
            continue
        dh = dyp[a:b] @ Wd[e]
        s = _sigmoid(g[a:b])
        dg[a:b] = dh * u[a:b] * s * (1.0 + g[a:b] * (1.0 - s))
        du[a:b] = dh * (g[a:b] * s)
        dxp[a:b] = dg[a:b] @ Wg[e] + du[a:b] @ Wu[e]
        dWd[e] = dyp[a:b].T @ h[a:b]
        dWg[e] = dg[a:b].T @ xp[a:b]
        dWu[e] = du[a:b].T @ xp[a:b]
    return {"dxp": dxp, "dg": dg, "du": du, "dWg": dWg, "dWu": dWu, "dWd": dWd}


# --------------------------------------------------------------------------
# Stage 5 (output reduction)
# --------------------------------------------------------------------------
def combine_fwd(yp, slot_row, topk_w) -> np.ndarray:
    """out[t] = sum over t's local slots, in slot order, of w[t,i] * yp[row(t,i)]."""
    T, k = slot_row.shape
    out = np.zeros((T, yp.shape[1]), dtype=yp.dtype)
    for i in range(k):
        rows = slot_row[:, i]
        m = rows >= 0
        out[m] += topk_w[m, i, None].astype(yp.dtype) * yp[rows[m]]
    return out


def combine_bwd(dout, yp, slot_row, topk_w):
    """dyp[row(t,i)] = w[t,i] * dout[t];  dgate[t,i] = <yp[row(t,i)], dout[t]> (0 if not local)."""
    T, k = slot_row.shape
    dyp = np.zeros_like(yp)
    dgate = np.zeros((T, k), dtype=yp.dtype)
    for i in range(k):
        rows = slot_row[:, i]
        m = rows >= 0
        dyp[rows[m]] = topk_w[m, i, None].astype(yp.dtype) * dout[m]
        dgate[m, i] = np.einsum("rh,rh->r", yp[rows[m]], dout[m])
    return dyp, dgate


# --------------------------------------------------------------------------
# The whole path
# --------------------------------------------------------------------------
def layer_fwd_bwd(inp: Dict[str, np.ndarray], k: int, e_begin: int, e_count: int,
                  renormalize: int = 1, dtype=np.float64) -> Dict[str, np.ndarray]:
    """All steps in order on one batch drawn by the workload generator.

    ``inp`` holds logits (fp32) and bf16 bit patterns x, dout, Wg, Wu, Wd.
    """
    x = decode_bf16(inp["x"], dtype)
    dout = decode_bf16(inp["dout"], dtype)
    Wg = decode_bf16(inp["Wg"], dtype)
    Wu = decode_bf16(inp["Wu"], dtype)
    Wd = decode_bf16(inp["Wd"], dtype)
    r: Dict[str, np.ndarray] = {}
    r["topk_idx"], r["topk_w"] = route(inp["logits"], k, renormalize, dtype)
    r["expert_offsets"], r["row_token"], r["slot_row"], r["xp"] = permute(
        x, r["topk_idx"], e_begin, e_count)
    r.update(expert_mlp_fwd(r["xp"], r["expert_offsets"], Wg, Wu, Wd))
    r["out"] = combine_fwd(r["yp"], r["slot_row"], r["topk_w"])
    r["dyp"], r["dgate"] = combine_bwd(dout, r["yp"], r["slot_row"], r["topk_w"])
    r.update(expert_mlp_bwd(r["dyp"], r["xp"], r["g"], r["u"], r["h"],
                            r["expert_offsets"], Wg, Wu, Wd))
    r["dx"] = permute_bwd(r["dxp"], r["slot_row"])
    return r
