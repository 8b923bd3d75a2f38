"""Pins for the expert MLP, combine and every backward step of the oracle
(Algorithm 1, Stages 4-5, and their derivatives)."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O


def random_topk(rng, T, E, k):
    return np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)


def draw(rng, T, d, E, k, f, scale=0.5):
    return dict(
        x=rng.standard_normal((T, d)),
        Wg=rng.standard_normal((E, f, d)) * scale,
        Wu=rng.standard_normal((E, f, d)) * scale,
        Wd=rng.standard_normal((E, d, f)) * scale,
        idx=random_topk(rng, T, E, k),
        w=rng.random((T, k)) + 0.1,
        dout=rng.standard_normal((T, d)),
    )


def oracle_chain(p, e_begin, e_count):
    """Run the oracle's steps on fp64 arrays (weights already sliced to the local range)."""
    off, rt, sr, xp = O.permute(p["x"], p["idx"], e_begin, e_count)
    sl = slice(e_begin, e_begin + e_count)
    Wg, Wu, Wd = p["Wg"][sl], p["Wu"][sl], p["Wd"][sl]
    fw = O.expert_mlp_fwd(xp, off, Wg, Wu, Wd)
    out = O.combine_fwd(fw["yp"], sr, p["w"])
    dyp, dgate = O.combine_bwd(p["dout"], fw["yp"], sr, p["w"])
    bw = O.expert_mlp_bwd(dyp, xp, fw["g"], fw["u"], fw["h"], off, Wg, Wu, Wd)
    dx = O.permute_bwd(bw["dxp"], sr)
    return dict(out=out, dgate=dgate, dx=dx, off=off, sr=sr, **fw, **bw, dyp=dyp)


def dense_definition_python(p):
    """out[t] = sum_i w[t,i] * MLP_{e(t,i)}(x[t]), token by token, scalar loops."""
    T, d = p["x"].shape
    k = p["idx"].shape[1]
    f = p["Wg"].shape[1]
    out = np.zeros((T, d))
    for t in range(T):
        for i in range(k):
            e = p["idx"][t, i]
            hvec = np.zeros(f)
            for j in range(f):
                gj = sum(p["Wg"][e, j, c] * p["x"][t, c] for c in range(d))
                uj = sum(p["Wu"][e, j, c] * p["x"][t, c] for c in range(d))
                hvec[j] = gj / (1.0 + np.exp(-gj)) * uj
            for c in range(d):
                out[t, c] += p["w"][t, i] * sum(p["Wd"][e, c, j] * hvec[j] for j in range(f))
    return out


def dense_definition_torch(p):
    """Same definition through torch CPU (fp64) with autograd; no permutation anywhere."""
    t64 = lambda a: torch.tensor(a, dtype=torch.float64, requires_grad=True)
    x, Wg, Wu, Wd, w = t64(p["x"]), t64(p["Wg"]), t64(p["Wu"]), t64(p["Wd"]), t64(p["w"])
    idx = torch.tensor(p["idx"], dtype=torch.long)
    T, k = idx.shape
    out = torch.zeros_like(x)
    for i in range(k):
        e = idx[:, i]
        g = torch.einsum("tfd,td->tf", Wg[e], x)
        u = torch.einsum("tfd,td->tf", Wu[e], x)
        h = torch.nn.functional.silu(g) * u
        out = out + w[:, i, None] * torch.einsum("tdf,tf->td", Wd[e], h)
    loss = (out * torch.tensor(p["dout"])).sum()
    loss.backward()
    return out.detach().numpy(), dict(dx=x.grad.numpy(), dWg=Wg.grad.numpy(), dWu=Wu.grad.numpy(),
                                      dWd=Wd.grad.numpy(), dgate=w.grad.numpy())


def test_forward_matches_scalar_dense_definition():
    rng = np.random.default_rng(0)
    p = draw(rng, T=6, d=4, E=3, k=2, f=5)
    r = oracle_chain(p, 0, 3)
    np.testing.assert_allclose(r["out"], dense_definition_python(p), rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("T,d,E,k,f", [(8, 4, 3, 2, 5), (33, 6, 8, 3, 7), (20, 5, 16, 8, 4)])
def test_forward_and_backward_match_library_autograd(T, d, E, k, f):
    rng = np.random.default_rng(T)
    p = draw(rng, T, d, E, k, f)
    r = oracle_chain(p, 0, E)
    out, grads = dense_definition_torch(p)
    np.testing.assert_allclose(r["out"], out, rtol=1e-11, atol=1e-12)
    for name in ("dx", "dWg", "dWu", "dWd", "dgate"):
        np.testing.assert_allclose(r[name], grads[name], rtol=1e-10, atol=1e-11, err_msg=name)


def test_backward_matches_finite_differences():
    rng = np.random.default_rng(3)
    T, d, E, k, f = 8, 4, 3, 2, 5
    p = draw(rng, T, d, E, k, f)
    r = oracle_chain(p, 0, E)

    def loss(q):
        return float((oracle_chain(q, 0, E)["out"] * q["dout"]).sum())

    eps = 1e-6
    for name, gname in (("x", "dx"), ("Wg", "dWg"), ("Wu", "dWu"), ("Wd", "dWd"), ("w", "dgate")):
        num = np.zeros_like(p[name])
        it = np.nditer(p[name], flags=["multi_index"])
        for _ in it:
            i = it.multi_index
            q = {key: (v.copy() if key == name else v) for key, v in p.items()}
            q[name][i] += eps
            up = loss(q)
            q[name][i] -= 2 * eps
            num[i] = (up - loss(q)) / (2 * eps)
        np.testing.assert_allclose(r[gname], num, rtol=2e-6, atol=2e-7, err_msg=gname)


def test_intermediate_gradients_by_autograd_on_the_grouped_form():
    """dyp, dxp, dg, du: leaves of a torch graph built on the oracle's own grouping."""
    rng = np.random.default_rng(4)
    T, d, E, k, f = 12, 5, 4, 2, 6
    p = draw(rng, T, d, E, k, f)
    r = oracle_chain(p, 0, E)
    off, sr = r["off"], r["sr"]
    tt = lambda a: torch.tensor(a, dtype=torch.float64, requires_grad=True)
    xp = tt(O.permute(p["x"], p["idx"], 0, E)[3])
    Wg, Wu, Wd = (torch.tensor(p[n]) for n in ("Wg", "Wu", "Wd"))
    g = torch.cat([xp[off[e]:off[e + 1]] @ Wg[e].T for e in range(E)])
    u = torch.cat([xp[off[e]:off[e + 1]] @ Wu[e].T for e in range(E)])
    g.retain_grad(); u.retain_grad()
    h = torch.nn.functional.silu(g) * u
    yp = torch.cat([h[off[e]:off[e + 1]] @ Wd[e].T for e in range(E)])
    yp.retain_grad()
    out = torch.zeros(T, d, dtype=torch.float64)
    w = torch.tensor(p["w"])
    for i in range(k):
        out = out + w[:, i, None] * yp[torch.tensor(sr[:, i], dtype=torch.long)]
    (out * torch.tensor(p["dout"])).sum().backward()
    np.testing.assert_allclose(r["dyp"], yp.grad.numpy(), rtol=1e-11, atol=1e-12)
    np.testing.assert_allclose(r["dg"], g.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(r["du"], u.grad.numpy(), rtol=1e-10, atol=1e-12)
    np.testing.assert_allclose(r["dxp"], xp.grad.numpy(), rtol=1e-10, atol=1e-12)


def test_single_expert_is_a_plain_swiglu_mlp():
    rng = np.random.default_rng(5)
    T, d, f = 17, 6, 9
    p = draw(rng, T, d, 1, 1, f)
    p["w"][:] = 1.0
    r = oracle_chain(p, 0, 1)
    x = torch.tensor(p["x"])
    ref = (torch.nn.functional.silu(x @ torch.tensor(p["Wg"][0]).T) * (x @ torch.tensor(p["Wu"][0]).T)) \
        @ torch.tensor(p["Wd"][0]).T
    np.testing.assert_allclose(r["out"], ref.numpy(), rtol=1e-12, atol=1e-13)
    assert np.array_equal(r["sr"][:, 0], np.arange(T))


def test_zero_down_weight_and_empty_experts():
    rng = np.random.default_rng(6)
    T, d, E, k, f = 30, 4, 6, 2, 5
    p = draw(rng, T, d, E, k, f)
    p["idx"] = random_topk(rng, T, 4, k)        # experts 4 and 5 get no token
    r = oracle_chain(p, 0, E)
    assert r["off"][4] == r["off"][5] == r["off"][6] == T * k
    for n in ("dWg", "dWu", "dWd"):
        assert np.all(r[n][4:] == 0.0) and np.any(r[n][:4] != 0.0)
    p["Wd"][:] = 0.0
    r0 = oracle_chain(p, 0, E)
    assert np.all(r0["out"] == 0.0) and np.all(r0["dx"] == 0.0) and np.all(r0["dgate"] == 0.0)


@pytest.mark.parametrize("EP", [2, 4])
def test_expert_parallel_partials_add_up(EP):
    """Each rank reduces its K_r local experts; the partial outputs sum to the
    EP=1 output (Section 3.1, Stage 5), and so do the partial input gradients."""
    rng = np.random.default_rng(7 + EP)
    T, d, E, k, f = 40, 5, 8, 3, 6
    p = draw(rng, T, d, E, k, f)
    full = oracle_chain(p, 0, E)
    NR = E // EP
    out = np.zeros_like(full["out"]); dx = np.zeros_like(full["dx"]); dgate = np.zeros_like(full["dgate"])
    rows = 0
    for r in range(EP):
        part = oracle_chain(p, r * NR, NR)
        out += part["out"]; dx += part["dx"]; dgate += part["dgate"]
        rows += part["off"][-1]
        sl = slice(r * NR, (r + 1) * NR)
        for n in ("dWg", "dWu", "dWd"):
            np.testing.assert_allclose(part[n], full[n][sl], rtol=1e-12, atol=1e-13)
        assert np.all((part["sr"] >= 0) == ((p["idx"] >= r * NR) & (p["idx"] < (r + 1) * NR)))
    assert rows == T * k
    np.testing.assert_allclose(out, full["out"], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dx, full["dx"], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(dgate, full["dgate"], rtol=1e-12, atol=1e-13)


def test_layer_entry_point_on_generated_inputs():
    """layer_fwd_bwd wires the steps in order on bf16-bit inputs; fp32 variant agrees with fp64."""
    from paper_2604_00785_amd import workloads as W
    for name in ("tiny", "skew"):
        cfg = W.CONFIGS[name]
        inp = W.make_inputs(cfg)
        r = O.layer_fwd_bwd(inp, cfg.k, 0, cfg.E)
        counts = np.diff(r["expert_offsets"])
        assert counts.sum() == cfg.T * cfg.k
        if name == "skew":
            assert counts.min() == 0 and counts[0] == counts.max()
        np.testing.assert_allclose(r["topk_w"].sum(1), 1.0, atol=1e-12)
        x = O.decode_bf16(inp["x"])
        assert np.array_equal(r["xp"], x[r["row_token"]])
        p = dict(x=x, Wg=O.decode_bf16(inp["Wg"]), Wu=O.decode_bf16(inp["Wu"]), Wd=O.decode_bf16(inp["Wd"]),
                 idx=r["topk_idx"], w=r["topk_w"], dout=O.decode_bf16(inp["dout"]))
        out, grads = dense_definition_torch(p)
        np.testing.assert_allclose(r["out"], out, rtol=1e-9, atol=1e-12)
        for n in ("dx", "dWg", "dWu", "dWd", "dgate"):
            np.testing.assert_allclose(r[n], grads[n], rtol=1e-8, atol=1e-12, err_msg=n)
        r32 = O.layer_fwd_bwd(inp, cfg.k, 0, cfg.E, dtype=np.float32)
        assert np.array_equal(r32["slot_row"], r["slot_row"])
        for n in ("out", "dx", "dWd"):
            assert np.abs(r32[n] - r[n]).max() <= 1e-4 * np.abs(r[n]).max()


@pytest.mark.parametrize("EP", [1, 2])
def test_gate_weights_may_be_folded_into_h(EP):
    """Stage 5 is linear in the experts' outputs, so the weight of a routed row may multiply h instead of yp.
    With hw = w h: the unweighted sum of hw.Wd^T rows is `out`; dWd = dout[token]^T hw; dh = w (dout[token].Wd);
    and the gate gradient is the row dot product of dout[token].Wd with h.  Checked on the oracle's own
    results (the HIP path has entry points that compute the layer this way)."""
    rng = np.random.default_rng(17 + EP)
    T, d, E, k, f = 23, 10, 6, 3, 7
    p = draw(rng, T, d, E, k, f)
    nl = E // EP
    for part in range(EP):
        eb = part * nl
        r = oracle_chain(p, eb, nl)
        off, sr = r["off"], r["sr"]
        R = int(off[-1])
        rows = sr[sr >= 0]
        w_row = np.zeros(R)
        w_row[rows] = p["w"][sr >= 0]
        tok = np.zeros(R, dtype=np.int64)
        tok[rows] = np.nonzero(sr >= 0)[0]
        Wd = p["Wd"][eb:eb + nl]
        hw = r["h"] * w_row[:, None]
        out = np.zeros((T, d))
        dWd = np.zeros_like(Wd)
        dgate_rows = np.zeros(R)
        for e in range(nl):
            a, b = int(off[e]), int(off[e + 1])
            ypw = hw[a:b] @ Wd[e].T
            np.testing.assert_allclose(ypw, r["yp"][a:b] * w_row[a:b, None], rtol=1e-12, atol=1e-14)
            np.add.at(out, tok[a:b], ypw)
            dg_rows = p["dout"][tok[a:b]]
            dWd[e] = dg_rows.T @ hw[a:b]
            dh0 = dg_rows @ Wd[e]
            dgate_rows[a:b] = (dh0 * r["h"][a:b]).sum(1)
            # dh = w dh0 is what the SwiGLU derivative starts from: compare through du = dh silu(g)
            silu = r["g"][a:b] / (1.0 + np.exp(-r["g"][a:b]))
            np.testing.assert_allclose(r["du"][a:b], (w_row[a:b, None] * dh0) * silu, rtol=1e-10, atol=1e-13)
        np.testing.assert_allclose(out, r["out"], rtol=1e-11, atol=1e-13)
        np.testing.assert_allclose(dWd, r["dWd"], rtol=1e-11, atol=1e-13)
        dgate = np.zeros((T, k))
        dgate[sr >= 0] = dgate_rows[rows]
        np.testing.assert_allclose(dgate, r["dgate"], rtol=1e-10, atol=1e-13)
