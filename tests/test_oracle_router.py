"""Pins for the oracle's router functions (Stage 1 of Algorithm 1 and its derivative): finite
differences, library autograd on the plain definition, closed forms and invariants."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O


def _gates(logits, idx, renorm):
    """The k gate weights for FIXED chosen experts, written out with scalar loops."""
    T, E = logits.shape
    k = idx.shape[1]
    w = np.zeros((T, k))
    for t in range(T):
        m = max(logits[t])
        den = sum(np.exp(logits[t, e] - m) for e in range(E))
        s = [np.exp(logits[t, idx[t, i]] - m) / den for i in range(k)]
        tot = sum(s) if renorm else 1.0
        for i in range(k):
            w[t, i] = s[i] / tot
    return w


@pytest.mark.parametrize("renorm", [0, 1])
@pytest.mark.parametrize("T,E,k", [(5, 6, 2), (3, 9, 4), (4, 4, 4), (2, 7, 1)])
def test_route_bwd_finite_differences(T, E, k, renorm):
    rng = np.random.default_rng(T * 31 + E + k)
    logits = rng.standard_normal((T, E)).astype(np.float32)
    idx, _ = O.route(logits, k, renorm)
    c = rng.standard_normal((T, k))
    got = O.route_bwd(logits, idx, c, renorm)
    eps = 1e-6
    fd = np.zeros((T, E))
    l64 = logits.astype(np.float64)
    for t in range(T):
        for e in range(E):
            lp, lm = l64.copy(), l64.copy()
            lp[t, e] += eps
            lm[t, e] -= eps
            fd[t, e] = ((_gates(lp, idx, renorm) * c).sum() - (_gates(lm, idx, renorm) * c).sum()) / (2 * eps)
    np.testing.assert_allclose(got, fd, rtol=1e-6, atol=1e-9)


@pytest.mark.parametrize("renorm", [0, 1])
def test_route_bwd_matches_library_autograd(renorm):
    rng = np.random.default_rng(7)
    T, E, k = 40, 16, 5
    logits = rng.standard_normal((T, E)).astype(np.float32)
    idx, w_ref = O.route(logits, k, renorm)
    c = rng.standard_normal((T, k))
    l = torch.tensor(logits, dtype=torch.float64, requires_grad=True)
    p = torch.softmax(l, dim=1)
    s = torch.gather(p, 1, torch.tensor(idx, dtype=torch.int64))
    w = s / s.sum(dim=1, keepdim=True) if renorm else s
    np.testing.assert_allclose(w.detach().numpy(), w_ref, rtol=1e-12)
    (w * torch.tensor(c)).sum().backward()
    np.testing.assert_allclose(O.route_bwd(logits, idx, c, renorm), l.grad.numpy(), rtol=1e-10, atol=1e-14)


def test_route_bwd_invariants_and_special_cases():
    rng = np.random.default_rng(3)
    T, E, k = 50, 12, 4
    logits = (rng.standard_normal((T, E)) * 3).astype(np.float32)
    idx, w = O.route(logits, k, 1)
    c = rng.standard_normal((T, k))
    for renorm in (0, 1):
        dl = O.route_bwd(logits, idx, c, renorm)
        # softmax does not see a common shift of a token's logits
        np.testing.assert_allclose(dl.sum(axis=1), 0.0, atol=1e-12)
    # renormalised gates sum to one, so a gradient that is the same for all k slots gives nothing
    dl = O.route_bwd(logits, idx, np.ones((T, k)) * 2.5, 1)
    np.testing.assert_allclose(dl, 0.0, atol=1e-12)
    # k = E: renormalising changes nothing (the probabilities already sum to one) and the result is the
    # softmax Jacobian applied to the gradient, placed by expert
    idxE, _ = O.route(logits, E, 1)
    cE = rng.standard_normal((T, E))
    by_expert = np.zeros((T, E))
    np.put_along_axis(by_expert, idxE.astype(np.int64), cE, axis=1)
    l64 = logits.astype(np.float64)
    p = np.exp(l64 - l64.max(1, keepdims=True))
    p /= p.sum(1, keepdims=True)
    jac = p * (by_expert - (by_expert * p).sum(1, keepdims=True))
    np.testing.assert_allclose(O.route_bwd(logits, idxE, cE, 1), jac, rtol=1e-9, atol=1e-13)
    np.testing.assert_allclose(O.route_bwd(logits, idxE, cE, 0), jac, rtol=1e-9, atol=1e-13)
    # experts that were not chosen still get a gradient (through the softmax denominator), of the sign
    # opposite to the chosen ones' weighted gradient
    dl = O.route_bwd(logits, idx, np.abs(c), 0)
    chosen = np.zeros((T, E), bool)
    np.put_along_axis(chosen, idx.astype(np.int64), True, axis=1)
    assert np.all(dl[~chosen] < 0)


def test_router_linear_and_its_derivative():
    rng = np.random.default_rng(11)
    T, d, E = 9, 7, 5
    x = rng.standard_normal((T, d))
    Wr = rng.standard_normal((E, d)).astype(np.float32)
    logits = O.router_logits(x, Wr)
    # scalar-loop definition
    for t in range(T):
        for e in range(E):
            assert abs(logits[t, e] - sum(x[t, j] * float(Wr[e, j]) for j in range(d))) < 1e-12
    dl = rng.standard_normal((T, E))
    dWr, dx = O.router_bwd(x, Wr, dl)
    xt = torch.tensor(x, requires_grad=True)
    wt = torch.tensor(Wr.astype(np.float64), requires_grad=True)
    ((xt @ wt.T) * torch.tensor(dl)).sum().backward()
    np.testing.assert_allclose(dWr, wt.grad.numpy(), rtol=1e-12)
    np.testing.assert_allclose(dx, xt.grad.numpy(), rtol=1e-12)
