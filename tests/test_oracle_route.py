"""Pins for oracle.route (Algorithm 1, Stage 1: Softmax then TopK)."""
import math

import numpy as np
import pytest

from oracle import moe_oracle as O


def brute_route(logits, k, renormalize):
    """Pure-Python selection by repeated maximum with the explicit tie rule."""
    T, E = logits.shape
    idx = [[0] * k for _ in range(T)]
    w = [[0.0] * k for _ in range(T)]
    for t in range(T):
        row = [float(v) for v in logits[t]]
        m = max(row)
        ex = [math.exp(v - m) for v in row]
        Z = math.fsum(ex)
        taken = set()
        for i in range(k):
            best = None
            for e in range(E):
                if e in taken:
                    continue
                if best is None or row[e] > row[best]:      # strict: lower id wins ties
                    best = e
            taken.add(best)
            idx[t][i] = best
            w[t][i] = ex[best] / Z
        if renormalize:
            s = math.fsum(w[t])
            w[t] = [v / s for v in w[t]]
    return np.array(idx, dtype=np.int32), np.array(w)


@pytest.mark.parametrize("T,E,k", [(7, 8, 2), (5, 64, 8), (3, 128, 8), (4, 5, 5), (6, 3, 1)])
@pytest.mark.parametrize("renorm", [0, 1])
def test_route_matches_brute_force(T, E, k, renorm):
    rng = np.random.default_rng(T * 1000 + E + k)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    # plant ties: duplicate some values inside rows
    logits[0, E - 1] = logits[0, 0]
    if E > 2:
        logits[1, 2] = logits[1, 1] = logits[1].max() + 1
    idx, w = O.route(logits, k, renorm)
    bidx, bw = brute_route(logits, k, renorm)
    assert np.array_equal(idx, bidx)
    np.testing.assert_allclose(w, bw, rtol=1e-12)


def test_route_invariants():
    rng = np.random.default_rng(1)
    T, E, k = 200, 64, 8
    logits = (rng.standard_normal((T, E)) * 3).astype(np.float32)
    idx, w = O.route(logits, k, 1)
    assert idx.dtype == np.int32 and idx.shape == (T, k) and w.shape == (T, k)
    assert idx.min() >= 0 and idx.max() < E
    for t in range(T):
        assert len(set(idx[t])) == k                      # k distinct experts per token
    assert np.all(np.diff(w, axis=1) <= 0)                # slots by decreasing gate
    np.testing.assert_allclose(w.sum(1), 1.0, atol=1e-12)  # renormalised gates sum to 1
    # every unselected logit is <= the smallest selected one
    sel_min = np.take_along_axis(logits, idx.astype(np.int64), 1).min(1)
    mask = np.ones((T, E), bool)
    np.put_along_axis(mask, idx.astype(np.int64), False, 1)
    assert np.all(np.where(mask, logits, -np.inf).max(1) <= sel_min)
    # paper-literal mode: the gates are entries of the full softmax
    idx0, w0 = O.route(logits, k, 0)
    assert np.array_equal(idx0, idx)
    l = logits.astype(np.float64)
    p = np.exp(l - l.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    np.testing.assert_allclose(w0, np.take_along_axis(p, idx.astype(np.int64), 1), rtol=1e-13)
    np.testing.assert_allclose(w0 / w0.sum(1, keepdims=True), w, rtol=1e-13)
    assert np.all(w0.sum(1) < 1.0)


def test_route_k_equals_E_is_full_softmax():
    rng = np.random.default_rng(2)
    logits = rng.standard_normal((9, 6)).astype(np.float32)
    idx, w = O.route(logits, 6, 0)
    from scipy.special import softmax
    p = softmax(logits.astype(np.float64), axis=1)
    assert np.array_equal(idx, np.argsort(-logits, axis=1, kind="stable"))
    np.testing.assert_allclose(w, np.take_along_axis(p, idx.astype(np.int64), 1), rtol=1e-12)
    np.testing.assert_allclose(w.sum(1), 1.0, atol=1e-12)


def test_route_ties():
    E, k = 8, 3
    logits = np.zeros((2, E), dtype=np.float32)
    logits[1, :] = 5.0
    idx, w = O.route(logits, k, 1)
    assert np.array_equal(idx, np.tile(np.arange(k, dtype=np.int32), (2, 1)))
    np.testing.assert_allclose(w, 1.0 / k)
    # -0.0 and +0.0 are equal logits: still a tie, lower id first
    z = np.array([[0.0, -0.0, -0.0, 0.0, -1.0]], dtype=np.float32)
    idx, _ = O.route(z, 4, 1)
    assert np.array_equal(idx[0], [0, 1, 2, 3])
    # large spread: no overflow, the top gate tends to 1
    big = np.array([[1000.0, -1000.0, 0.0, 999.0]], dtype=np.float32)
    idx, w = O.route(big, 2, 0)
    assert np.array_equal(idx[0], [0, 3])
    np.testing.assert_allclose(w[0], [1 / (1 + math.exp(-1)), math.exp(-1) / (1 + math.exp(-1))], rtol=1e-12)
