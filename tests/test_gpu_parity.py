"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.  Integer results bit-exact; floating point within
max|d|/max|ref| <= 2e-2 per tensor (bf16 storage, fp32 accumulation)."""
import numpy as np
import pytest
import torch

from oracle import moe_oracle as O
from paper_2604_00785_amd import binding as B
from paper_2604_00785_amd import workloads as W

import gpu_harness as H

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev_i32(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).to(DEV)


def random_topk(rng, T, E, k):
    return np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)


# ----------------------------------------------------------------------------- route
@pytest.mark.parametrize("T,E,k", [(256, 8, 2), (1000, 64, 8), (777, 128, 8), (50, 5, 5), (130, 100, 7),
                                   (64, 300, 70), (33, 512, 9), (1, 64, 8), (5, 1, 1)])
@pytest.mark.parametrize("renorm", [0, 1])
def test_route(T, E, k, renorm):
    print(f"route T={T} E={E} k={k} renorm={renorm}", flush=True)
    rng = np.random.default_rng(T + E + k)
    logits = (rng.standard_normal((T, E)) * 2).astype(np.float32)
    # ties: coarse values in some rows, all-equal rows, signed zeros
    logits[::7] = np.round(logits[::7])
    logits[3 % T] = 1.5
    if T > 4:
        logits[4] = np.where(rng.random(E) < 0.5, 0.0, -0.0).astype(np.float32)
    idx = torch.zeros(T, k, dtype=torch.int32, device=DEV)
    w = torch.zeros(T, k, dtype=torch.float32, device=DEV)
    B.moe_route(torch.from_numpy(logits).to(DEV), k, renorm, idx, w)
    torch.cuda.synchronize()
    ridx, rw = O.route(logits, k, renorm)
    assert np.array_equal(idx.cpu().numpy(), ridx)
    np.testing.assert_allclose(w.cpu().numpy(), rw, rtol=H.GATE_TOL)


# ----------------------------------------------------------------------------- permute
@pytest.mark.parametrize("T,E,k,d,eb,ec", [
    (256, 8, 2, 128, 0, 8), (1000, 64, 8, 256, 0, 64), (1000, 64, 8, 64, 16, 8), (513, 128, 8, 2048, 0, 128),
    (129, 12, 5, 4096, 3, 7), (7, 4, 1, 8, 0, 4), (4096, 512, 4, 72, 0, 512), (3000, 16, 4, 1032, 0, 16),
    (20000, 64, 8, 8, 0, 64),       # more than 256 * 256 pairs: chunks of several 256-pair units
    (9000, 300, 8, 8, 10, 280)])    # more than 128 local experts: at most 128 chunks, two table columns per thread
def test_permute(T, E, k, d, eb, ec):
    print(f"permute T={T} E={E} k={k} d={d} local=[{eb},{eb+ec})", flush=True)
    rng = np.random.default_rng(T * 3 + E)
    # expert eb+1 is never chosen when there are enough others: an empty local group
    pool = np.array([e for e in range(E) if e != eb + 1 or E <= 4])
    idx = np.stack([pool[rng.permutation(len(pool))[:k]] for _ in range(T)]).astype(np.int32)
    xb = W.f32_to_bf16_bits(rng.standard_normal((T, d)).astype(np.float32))
    x = H.bf16_to_dev(xb)
    R_cap = T * k
    off = torch.full((ec + 1,), -7, dtype=torch.int32, device=DEV)
    rt = torch.full((R_cap,), -7, dtype=torch.int32, device=DEV)
    sr = torch.full((T, k), -7, dtype=torch.int32, device=DEV)
    xp = torch.zeros(R_cap, d, dtype=torch.bfloat16, device=DEV)
    ws = torch.zeros(max(B.moe_permute_workspace_bytes(T, k, ec), 16), dtype=torch.uint8, device=DEV)
    B.moe_permute(x, dev_i32(idx), E, eb, ec, off, rt, sr, xp, ws)
    torch.cuda.synchronize()
    roff, rrt, rsr, rxp = O.permute(O.decode_bf16(xb), idx, eb, ec)
    R = int(roff[-1])
    assert np.array_equal(off.cpu().numpy(), roff)
    assert np.array_equal(sr.cpu().numpy(), rsr)
    assert np.array_equal(rt.cpu().numpy()[:R], rrt)
    assert np.all(rt.cpu().numpy()[R:] == -7)          # rows past R are left untouched
    assert np.array_equal(H.bf16_from_dev(xp)[:R], rxp)
    # twice the same call: same bits (no atomics, no races)
    off2, rt2, sr2 = torch.zeros_like(off), torch.zeros_like(rt), torch.zeros_like(sr)
    B.moe_permute(x, dev_i32(idx), E, eb, ec, off2, rt2, sr2, xp, ws)
    torch.cuda.synchronize()
    assert torch.equal(off, off2) and torch.equal(sr, sr2) and torch.equal(rt[:R], rt2[:R])


# ----------------------------------------------------------------------------- route + permute in one call
@pytest.mark.parametrize("T,E,k,eb,ec", [
    (256, 8, 2, 0, 8), (1000, 64, 8, 0, 64), (1000, 64, 8, 16, 8), (777, 128, 8, 0, 128), (50, 5, 5, 1, 3),
    (130, 100, 7, 0, 100), (64, 300, 70, 20, 200), (33, 512, 9, 0, 512), (1, 64, 8, 0, 64), (5, 1, 1, 0, 1),
    (8192, 64, 8, 0, 64),           # the headline shape: two passes of 16 tokens per workgroup
    (20000, 64, 8, 8, 48),          # several passes per workgroup, a last chunk that is not full
    (4100, 128, 16, 0, 128)])
@pytest.mark.parametrize("renorm,gate", [(0, False), (1, True)])
def test_route_permute_one_call(T, E, k, eb, ec, renorm, gate):
    print(f"route_permute T={T} E={E} k={k} local=[{eb},{eb+ec}) renorm={renorm} gate={gate}", flush=True)
    rng = np.random.default_rng(T + 5 * E + k)
    logits = (rng.standard_normal((T, E)) * 2).astype(np.float32)
    logits[::7] = np.round(logits[::7])          # ties
    d = 16
    xb = W.f32_to_bf16_bits(rng.standard_normal((T, d)).astype(np.float32))
    x, lg = H.bf16_to_dev(xb), torch.from_numpy(logits).to(DEV)
    R_cap = T * k
    mk = lambda shape, dt: torch.full(shape, -7, dtype=dt, device=DEV)
    idx, w = mk((T, k), torch.int32), mk((T, k), torch.float32)
    off, rt, sr = mk((ec + 1,), torch.int32), mk((R_cap,), torch.int32), mk((T, k), torch.int32)
    rw = mk((R_cap,), torch.float32) if gate else None
    xp = None if gate else torch.zeros(R_cap, d, dtype=torch.bfloat16, device=DEV)
    ws = torch.full((max(B.moe_permute_workspace_bytes(T, k, ec), 16),), 0x5A, dtype=torch.uint8, device=DEV)
    B.moe_route_permute(lg, None if gate else x, k, renorm, eb, ec, idx, w, off, rt, sr, rw, xp, ws)
    torch.cuda.synchronize()
    ridx, rwts = O.route(logits, k, renorm)
    roff, rrt, rsr, rxp = O.permute(O.decode_bf16(xb), ridx, eb, ec)
    R = int(roff[-1])
    assert np.array_equal(idx.cpu().numpy(), ridx)
    np.testing.assert_allclose(w.cpu().numpy(), rwts, rtol=H.GATE_TOL)
    assert np.array_equal(off.cpu().numpy(), roff)
    assert np.array_equal(sr.cpu().numpy(), rsr)
    assert np.array_equal(rt.cpu().numpy()[:R], rrt)
    assert np.all(rt.cpu().numpy()[R:] == -7)
    if gate:
        got_w = w.cpu().numpy()
        want = np.zeros(R, dtype=np.float32)
        want[rsr[rsr >= 0]] = got_w[rsr >= 0]
        assert np.array_equal(rw.cpu().numpy()[:R], want)     # a copy of the gate weights, row by row
    else:
        assert np.array_equal(H.bf16_from_dev(xp)[:R], rxp)
    # the two-call form gives the same bits
    idx2, w2 = mk((T, k), torch.int32), mk((T, k), torch.float32)
    off2, rt2, sr2 = mk((ec + 1,), torch.int32), mk((R_cap,), torch.int32), mk((T, k), torch.int32)
    B.moe_route(lg, k, renorm, idx2, w2)
    B.moe_permute(x, idx2, E, eb, ec, off2, rt2, sr2, None, ws)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(w, w2)
    assert torch.equal(off, off2) and torch.equal(sr, sr2) and torch.equal(rt[:R], rt2[:R])


@pytest.mark.parametrize("T,E,k,eb,ec", [(3000, 96, 6, 8, 8), (8192, 64, 8, 0, 64), (700, 16, 2, 0, 16), (24576, 96, 6, 88, 8)])
def test_route_permute_with_a_large_workspace(T, E, k, eb, ec):
    """A workspace beyond the minimum lets the routing kernel use short chunks (one pass of tokens per workgroup,
    fewer than 256 pairs when k is small): same results."""
    print(f"route_permute, 4 MiB workspace: T={T} E={E} k={k} local=[{eb},{eb+ec})", flush=True)
    rng = np.random.default_rng(T + E)
    logits = (rng.standard_normal((T, E)) * 2).astype(np.float32)
    logits[::5] = np.round(logits[::5])
    lg = torch.from_numpy(logits).to(DEV)
    mk = lambda shape, dt: torch.full(shape, -7, dtype=dt, device=DEV)
    idx, w = mk((T, k), torch.int32), mk((T, k), torch.float32)
    off, rt, sr = mk((ec + 1,), torch.int32), mk((T * k,), torch.int32), mk((T, k), torch.int32)
    rw = mk((T * k,), torch.float32)
    ws = torch.full((4 << 20,), 0xA5, dtype=torch.uint8, device=DEV)
    B.moe_route_permute(lg, None, k, 1, eb, ec, idx, w, off, rt, sr, rw, None, ws)
    torch.cuda.synchronize()
    ridx, rwts = O.route(logits, k, 1)
    roff, rrt, rsr, _ = O.permute(np.zeros((T, 1)), ridx, eb, ec)
    R = int(roff[-1])
    assert np.array_equal(idx.cpu().numpy(), ridx)
    np.testing.assert_allclose(w.cpu().numpy(), rwts, rtol=H.GATE_TOL)
    assert np.array_equal(off.cpu().numpy(), roff)
    assert np.array_equal(sr.cpu().numpy(), rsr)
    assert np.array_equal(rt.cpu().numpy()[:R], rrt)


# ----------------------------------------------------------------------------- combine (+bwd), permute_bwd
@pytest.mark.parametrize("T,E,k,d,eb,ec", [(256, 8, 2, 128, 0, 8), (500, 64, 8, 2048, 0, 64), (300, 16, 4, 4096, 4, 8),
                                           (77, 6, 3, 264, 0, 6)])
def test_combine_and_backward(T, E, k, d, eb, ec):
    print(f"combine T={T} E={E} k={k} d={d}", flush=True)
    rng = np.random.default_rng(T + d)
    idx = random_topk(rng, T, E, k)
    _, _, rsr, _ = O.permute(np.zeros((T, 1)), idx, eb, ec)
    R_cap = T * k
    ypb = W.f32_to_bf16_bits(rng.standard_normal((R_cap, d)).astype(np.float32))
    doutb = W.f32_to_bf16_bits(rng.standard_normal((T, d)).astype(np.float32))
    w = rng.random((T, k)).astype(np.float32)
    yp, dout, sr, wt = H.bf16_to_dev(ypb), H.bf16_to_dev(doutb), dev_i32(rsr), torch.from_numpy(w).to(DEV)
    out = torch.full((T, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    dx = torch.full((T, d), float("nan"), dtype=torch.bfloat16, device=DEV)
    dyp = torch.zeros(R_cap, d, dtype=torch.bfloat16, device=DEV)
    dgate = torch.full((T, k), float("nan"), dtype=torch.float32, device=DEV)
    B.moe_unpermute_combine(yp, sr, wt, out)
    B.moe_permute_bwd(yp, sr, dx)
    B.moe_unpermute_combine_bwd(dout, yp, sr, wt, dyp, dgate)
    torch.cuda.synchronize()
    ypf, doutf, wf = O.decode_bf16(ypb), O.decode_bf16(doutb), w.astype(np.float64)
    H.assert_close(H.bf16_from_dev(out), O.combine_fwd(ypf, rsr, wf), "out", 1e-2)
    H.assert_close(H.bf16_from_dev(dx), O.permute_bwd(ypf, rsr), "dx", 1e-2)
    rdyp, rdgate = O.combine_bwd(doutf, ypf, rsr, wf)
    used = np.zeros(R_cap, bool)
    used[rsr[rsr >= 0]] = True
    H.assert_close(H.bf16_from_dev(dyp)[used], rdyp[used], "dyp", 1e-2)
    assert np.all(H.bf16_from_dev(dyp)[~used] == 0)          # rows of no local slot are not written
    H.assert_close(dgate.cpu().numpy().astype(np.float64), rdgate, "dgate", 1e-4)


def test_permute_then_combine_is_identity():
    T, E, k, d = 512, 16, 4, 512
    rng = np.random.default_rng(9)
    idx = random_topk(rng, T, E, k)
    xb = W.f32_to_bf16_bits(rng.standard_normal((T, d)).astype(np.float32))
    buf = B.MoELayerBuffers(T, d, E, k, 64)
    x = H.bf16_to_dev(xb)
    B.moe_permute(x, dev_i32(idx), E, 0, E, buf.expert_offsets, buf.row_token, buf.slot_row, buf.xp, buf.ws)
    w = torch.full((T, k), 1.0 / k, dtype=torch.float32, device=DEV)
    B.moe_unpermute_combine(buf.xp, buf.slot_row, w, buf.out)
    torch.cuda.synchronize()
    assert torch.equal(buf.out.view(torch.int16), x.view(torch.int16))


# ----------------------------------------------------------------------------- grouped GEMMs, isolated
@pytest.mark.parametrize("counts,d,f", [
    ([64, 64, 64, 64], 128, 256),                 # whole tiles only partly filled
    ([300, 0, 5, 257, 256, 1, 0, 700], 192, 320),  # ragged rows and columns, empty experts
    ([1100, 900], 512, 128),                      # several row tiles per expert
    ([0, 0, 40], 64, 64),                         # leading empty experts, minimum sizes
    ([70, 1, 63, 64, 65, 128, 320, 330, 449], 64, 64),   # one reduction step forward; 1..8 steps in the weight gradients
    ([130, 130, 130], 320, 448),                  # 5 and 7 reduction steps: one and more rounds of the tile ring
    ([257, 511], 384, 704),                       # 6 and 11 steps, rows just past a tile boundary
    ([3] * 130, 64, 128),                         # more experts than a lane keeps in registers: per-tile prefix sums
    ([300 if e % 9 == 0 else 7 for e in range(100)], 64, 128),   # two experts per lane, mixed tile counts
])
def test_grouped_gemm_fwd_bwd_isolated(counts, d, f):
    print(f"gemm counts={counts} d={d} f={f}", flush=True)
    rng = np.random.default_rng(sum(counts) + d + f)
    E = len(counts)
    off = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    R = int(off[-1])
    R_cap = R + 37                                   # capacity beyond R must stay untouched
    mk = lambda shape, s: W.f32_to_bf16_bits((rng.standard_normal(shape) * s).astype(np.float32))
    xpb, dypb = mk((R_cap, d), 1.0), mk((R_cap, d), 1.0)
    Wgb, Wub, Wdb = mk((E, f, d), 0.05), mk((E, f, d), 0.05), mk((E, d, f), 0.05)
    xp, dyp = H.bf16_to_dev(xpb), H.bf16_to_dev(dypb)
    Wg, Wu, Wd = H.bf16_to_dev(Wgb), H.bf16_to_dev(Wub), H.bf16_to_dev(Wdb)
    nanbf = lambda *s: torch.full(s, float("nan"), dtype=torch.bfloat16, device=DEV)
    g, u, h, yp, dxp = nanbf(R_cap, f), nanbf(R_cap, f), nanbf(R_cap, f), nanbf(R_cap, d), nanbf(R_cap, d)
    dWg, dWu, dWd = nanbf(E, f, d), nanbf(E, f, d), nanbf(E, d, f)
    ws = torch.zeros(B.moe_grouped_gemm_bwd_workspace_bytes(R_cap, f), dtype=torch.uint8, device=DEV)
    offd = dev_i32(off)
    B.moe_grouped_gemm_fwd(xp, offd, Wg, Wu, Wd, g, u, h, yp)
    torch.cuda.synchronize()
    dec = O.decode_bf16
    fw = O.expert_mlp_fwd(dec(xpb)[:R], off, dec(Wgb), dec(Wub), dec(Wdb))
    got = {n: H.bf16_from_dev(t) for n, t in (("g", g), ("u", u), ("h", h), ("yp", yp))}
    for n in ("g", "u", "h", "yp"):
        H.assert_close(got[n][:R], fw[n], n)
        assert np.all(np.isnan(got[n][R:])), f"{n}: rows beyond R were written"
    # backward from the GPU's own saved activations (what a training step does)
    B.moe_grouped_gemm_bwd(dyp, xp, g, u, h, offd, Wg, Wu, Wd, dxp, dWg, dWu, dWd, ws)
    torch.cuda.synchronize()
    bw = O.expert_mlp_bwd(dec(dypb)[:R], dec(xpb)[:R], got["g"][:R], got["u"][:R], got["h"][:R], off,
                          dec(Wgb), dec(Wub), dec(Wdb))
    gdxp = H.bf16_from_dev(dxp)
    H.assert_close(gdxp[:R], bw["dxp"], "dxp")
    assert np.all(np.isnan(gdxp[R:]))
    # the two intermediate gradients the workspace holds on return: dg at its start, du half way in
    half = ws.numel() // 2
    for n, at in (("dg", 0), ("du", half)):
        t = ws[at:at + R_cap * f * 2].view(torch.bfloat16).view(R_cap, f)
        H.assert_close(H.bf16_from_dev(t)[:R], bw[n], n)
    for n, t in (("dWg", dWg), ("dWu", dWu), ("dWd", dWd)):
        gw = H.bf16_from_dev(t)
        for e in range(E):
            if counts[e] == 0:
                assert np.all(gw[e] == 0.0), f"{n}[{e}] must be zero"
            else:
                H.assert_close(gw[e], bw[n][e], f"{n}[{e}]")


@pytest.mark.parametrize("seed", range(8))
def test_grouped_gemm_random_shapes(seed):
    """Seeded random expert counts and widths: whole and ragged row tiles, experts whose tile count fills a whole
    run of tiles next to ones that do not, empty experts, one to 140 experts."""
    rng = np.random.default_rng(1000 + seed)
    E = int(rng.choice([1, 2, 7, 33, 64, 65, 100, 128, 129, 140]))
    d = int(rng.choice([64, 128, 192, 256, 512]))
    f = int(rng.choice([64, 128, 256, 320, 512]))
    kinds = rng.integers(0, 5, size=E)
    counts = [int({0: 0, 1: 256, 2: rng.integers(1, 40), 3: rng.integers(250, 270), 4: rng.integers(500, 530)}[k]) for k in kinds]
    if E > 64:
        counts = [min(c, 40) if i % 5 else c for i, c in enumerate(counts)]     # keep the total small
    if sum(counts) == 0:
        counts[0] = 17
    test_grouped_gemm_fwd_bwd_isolated(counts, d, f)


# ----------------------------------------------------------------------------- whole path, small configs
@pytest.mark.parametrize("name", ["tiny", "skew"])
def test_layer_small_configs(name):
    print(f"layer {name}", flush=True)
    cfg = W.CONFIGS[name]
    inp = W.make_inputs(cfg)
    res = H.run_layer(cfg, inp)
    ref = O.layer_fwd_bwd(inp, cfg.k, cfg.e_begin, cfg.n_local, cfg.renormalize)
    if name == "skew":
        assert np.diff(ref["expert_offsets"]).min() == 0
    H.compare_layer(res, ref, cfg.n_local)


@pytest.mark.parametrize("T,d,E,k,f,eb,ec,renorm", [
    (700, 192, 6, 3, 320, 0, 6, 1),       # ragged in every dimension
    (2048, 256, 16, 4, 128, 4, 8, 0),     # expert-parallel share, gates not renormalised
    (1500, 128, 4, 2, 64, 0, 4, 1),       # several row tiles per expert
    (200, 128, 128, 70, 64, 0, 128, 1),   # more than 64 slots per token, many experts with few rows
    (64, 64, 300, 9, 64, 100, 150, 1),    # wide expert range, most experts empty
])
def test_layer_ragged_shapes(T, d, E, k, f, eb, ec, renorm):
    print(f"layer T={T} d={d} E={E} k={k} f={f} local=[{eb},{eb+ec}) renorm={renorm}", flush=True)
    cfg = W.MoEConfig("custom", T=T, d=d, E=E, k=k, f=f, e_begin=eb, e_count=ec, renormalize=renorm, seed=T)
    inp = W.make_inputs(cfg)
    res = H.run_layer(cfg, inp)
    ref = O.layer_fwd_bwd(inp, k, eb, ec, renorm)
    H.compare_layer(res, ref, ec)


@pytest.mark.parametrize("seed", range(6))
def test_layer_random_shapes(seed):
    """Seeded random layer shapes and local expert ranges through each of the three forms of the path."""
    rng = np.random.default_rng(77 + seed)
    E = int(rng.choice([3, 8, 16, 64, 100, 128, 200]))
    k = int(rng.integers(1, min(E, 8) + 1))
    T = int(rng.choice([37, 256, 600, 1111]))    # (a single token is its own test: one ill-conditioned dot product
                                                 # is no basis for a relative bound)
    d, f = int(rng.choice([64, 128, 192])), int(rng.choice([64, 128, 320]))
    eb = int(rng.integers(0, E))
    ec = int(rng.integers(1, min(E - eb, 150) + 1))
    renorm = int(rng.integers(0, 2))
    mode = [dict(), dict(gather=True), dict(fold=True)][seed % 3]
    print(f"layer T={T} d={d} E={E} k={k} f={f} local=[{eb},{eb+ec}) renorm={renorm} {mode}", flush=True)
    cfg = W.MoEConfig("custom", T=T, d=d, E=E, k=k, f=f, e_begin=eb, e_count=ec, renormalize=renorm, seed=500 + seed)
    inp = W.make_inputs(cfg)
    res = H.run_layer(cfg, inp, **mode)
    ref = O.layer_fwd_bwd(inp, k, eb, ec, renorm)
    H.compare_layer(res, ref, ec)


@pytest.mark.parametrize("T,d,E,k,f,eb,ec,renorm", [
    (256, 128, 8, 2, 256, 0, 8, 1),       # the tiny config's shape
    (700, 192, 6, 3, 320, 0, 6, 1),       # ragged in every dimension
    (2048, 256, 16, 4, 128, 4, 8, 0),     # expert-parallel share
    (1500, 128, 4, 2, 64, 0, 4, 1),       # several row tiles and several reduction steps per expert
    (64, 64, 300, 9, 64, 100, 150, 1),    # most experts empty, experts with a single row
    (3000, 512, 3, 1, 192, 0, 3, 1),      # about 1000 rows per expert: many reduction steps in the weight gradients
])
def test_layer_gathered_rows(T, d, E, k, f, eb, ec, renorm):
    """The products that read x through row_token instead of a materialised xp: against the oracle,
    and bit for bit against the xp path (same operands, same order of arithmetic)."""
    print(f"gathered layer T={T} d={d} E={E} k={k} f={f} local=[{eb},{eb+ec}) renorm={renorm}", flush=True)
    cfg = W.MoEConfig("custom", T=T, d=d, E=E, k=k, f=f, e_begin=eb, e_count=ec, renormalize=renorm, seed=T + 1)
    inp = W.make_inputs(cfg)
    res = H.run_layer(cfg, inp, gather=True)
    assert "xp" not in res
    ref = O.layer_fwd_bwd(inp, k, eb, ec, renorm)
    H.compare_layer(res, ref, ec)
    plain = H.run_layer(cfg, inp)
    R = int(ref["expert_offsets"][-1])
    for n in ("g", "u", "h", "yp", "dyp", "dxp"):
        assert np.array_equal(res[n][:R], plain[n][:R]), n
    for n in ("out", "dx", "dgate", "dWg", "dWu", "dWd"):
        assert np.array_equal(res[n], plain[n]), n


@pytest.mark.parametrize("T,d,E,k,f,eb,ec,renorm", [
    (256, 128, 8, 2, 256, 0, 8, 1),       # the tiny config's shape
    (700, 192, 6, 3, 320, 0, 6, 1),       # ragged in every dimension
    (2048, 256, 16, 4, 128, 4, 8, 0),     # expert-parallel share, no renormalisation
    (1500, 128, 4, 2, 64, 0, 4, 1),       # several row tiles and several reduction steps per expert
    (64, 64, 300, 9, 64, 100, 150, 1),    # most experts empty, experts with a single row
    (3000, 512, 3, 1, 192, 0, 3, 1),      # about 1000 rows per expert: many reduction steps in the weight gradients
    (1, 64, 4, 2, 64, 0, 4, 1),           # a single token
    (300, 64, 130, 5, 64, 0, 130, 1),     # more than 64 local experts (tile lookup in two passes), one column strip
    (513, 320, 70, 6, 192, 3, 67, 0),     # odd sizes, a local slice of more than 64 experts, no renormalisation
    (2000, 256, 2, 2, 448, 0, 2, 1),      # two big experts: many row tiles each, seven column strips
])
def test_layer_folded_gate_weights(T, d, E, k, f, eb, ec, renorm):
    """The path that folds the gate weights into h and takes dgate from the backward product of the down
    projection: against the oracle (hw = w h, ypw = w yp, everything else unchanged)."""
    print(f"folded layer T={T} d={d} E={E} k={k} f={f} local=[{eb},{eb+ec}) renorm={renorm}", flush=True)
    cfg = W.MoEConfig("custom", T=T, d=d, E=E, k=k, f=f, e_begin=eb, e_count=ec, renormalize=renorm, seed=T + 3)
    inp = W.make_inputs(cfg)
    res = H.run_layer(cfg, inp, fold=True)
    assert "xp" not in res and "dyp" not in res
    ref = O.layer_fwd_bwd(inp, k, eb, ec, renorm)
    H.compare_layer(res, ref, ec)
    # g and u do not depend on the gate weights: bit for bit those of the gathered path
    plain = H.run_layer(cfg, inp, gather=True)
    R = int(ref["expert_offsets"][-1])
    for n in ("g", "u"):
        assert np.array_equal(res[n][:R], plain[n][:R]), n


def test_layer_folded_without_local_rows():
    """No token routed to the local experts: zeros everywhere, through the folded path."""
    cfg = W.MoEConfig("custom", T=192, d=128, E=8, k=2, f=64, e_begin=6, e_count=2, seed=3)
    inp = W.make_inputs(cfg)
    inp["logits"][:, 6:] = -50.0          # experts 6 and 7 are never among the top 2
    res = H.run_layer(cfg, inp, fold=True)
    assert int(res["expert_offsets"][-1]) == 0
    for n in ("out", "dx", "dgate", "dWg", "dWu", "dWd"):
        assert np.all(res[n] == 0.0), n


# ----------------------------------------------------------------------------- router and Stage-1 backward
@pytest.mark.parametrize("T,d,E", [(256, 128, 8), (1000, 2048, 64), (77, 64, 100), (33, 48, 5), (4096, 256, 300)])
def test_router_fwd(T, d, E):
    print(f"router_fwd T={T} d={d} E={E}", flush=True)
    rng = np.random.default_rng(T + d + E)
    xb = W.f32_to_bf16_bits(rng.standard_normal((T, d)).astype(np.float32))
    Wr = (rng.standard_normal((E, d)) * 0.05).astype(np.float32)
    logits = torch.full((T, E), float("nan"), dtype=torch.float32, device=DEV)
    B.moe_router_fwd(H.bf16_to_dev(xb), torch.from_numpy(Wr).to(DEV), logits)
    torch.cuda.synchronize()
    ref = O.router_logits(O.decode_bf16(xb), Wr)
    got = logits.cpu().numpy().astype(np.float64)
    # exact products, fp32 accumulation over d terms: error ~ sqrt(d) * 2^-24 * |terms|
    scale = np.abs(ref).max()
    assert np.abs(got - ref).max() <= 2e-6 * scale * max(1.0, np.sqrt(d) / 8)


@pytest.mark.parametrize("T,E,k", [(256, 8, 2), (1000, 64, 8), (130, 100, 7), (64, 300, 70), (5, 1, 1), (33, 512, 9)])
@pytest.mark.parametrize("renorm", [0, 1])
def test_route_bwd(T, E, k, renorm):
    print(f"route_bwd T={T} E={E} k={k} renorm={renorm}", flush=True)
    rng = np.random.default_rng(T * 7 + E + k)
    logits = (rng.standard_normal((T, E)) * 2).astype(np.float32)
    idx, _ = O.route(logits, k, renorm)
    dgate = rng.standard_normal((T, k)).astype(np.float32)
    dl = torch.full((T, E), float("nan"), dtype=torch.float32, device=DEV)
    B.moe_route_bwd(torch.from_numpy(logits).to(DEV), dev_i32(idx), torch.from_numpy(dgate).to(DEV), renorm, dl)
    torch.cuda.synchronize()
    ref = O.route_bwd(logits, idx, dgate, renorm)
    got = dl.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(got))
    assert np.abs(got - ref).max() <= 2e-5 * max(np.abs(ref).max(), 1e-30)


@pytest.mark.parametrize("T,d,E", [(256, 128, 8), (1000, 2048, 64), (300, 64, 100), (33, 48, 5), (2100, 256, 130),
                                   (500, 192, 72), (70, 512, 136)])
def test_router_bwd(T, d, E):
    print(f"router_bwd T={T} d={d} E={E}", flush=True)
    rng = np.random.default_rng(T + 3 * d + E)
    xb = W.f32_to_bf16_bits(rng.standard_normal((T, d)).astype(np.float32))
    dx0b = W.f32_to_bf16_bits(rng.standard_normal((T, d)).astype(np.float32))
    Wr = (rng.standard_normal((E, d)) * 0.05).astype(np.float32)
    dl = (rng.standard_normal((T, E)) * 0.1).astype(np.float32)
    dx = H.bf16_to_dev(dx0b).clone()
    dWr = torch.full((E, d), float("nan"), dtype=torch.float32, device=DEV)
    ws = torch.zeros(B.moe_router_bwd_workspace_bytes(T, d, E), dtype=torch.uint8, device=DEV)
    B.moe_router_bwd(H.bf16_to_dev(xb), torch.from_numpy(Wr).to(DEV), torch.from_numpy(dl).to(DEV), dx, dWr, ws)
    torch.cuda.synchronize()
    rdWr, rdx = O.router_bwd(O.decode_bf16(xb), Wr, dl.astype(np.float64))
    got = dWr.cpu().numpy().astype(np.float64)
    assert np.abs(got - rdWr).max() <= 1e-5 * np.abs(rdWr).max()
    H.assert_close(H.bf16_from_dev(dx), O.decode_bf16(dx0b) + rdx, "dx", 1e-2)
    # the same call again gives the same dWr bits (fixed reduction order, no atomics)
    dWr2 = torch.zeros_like(dWr)
    B.moe_router_bwd(H.bf16_to_dev(xb), torch.from_numpy(Wr).to(DEV), torch.from_numpy(dl).to(DEV), dx, dWr2, ws)
    torch.cuda.synchronize()
    assert torch.equal(dWr, dWr2)


@pytest.mark.parametrize("gather", [False, True, "fold"])
def test_drop_in_block_router_to_gradients(gather):
    """Router -> route on the device's own logits -> ... -> dgate -> dlogits -> dWr, dx: the chain a
    training step runs, against the oracle fed with the same (device) logits."""
    cfg = W.MoEConfig("custom", T=512, d=128, E=16, k=4, f=64, seed=5)
    inp = W.make_inputs(cfg)
    buf = B.MoELayerBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, gather=bool(gather), fold=(gather == "fold"))
    x, dout = H.bf16_to_dev(inp["x"]), H.bf16_to_dev(inp["dout"])
    Wg, Wu, Wd = (H.bf16_to_dev(inp[n]) for n in ("Wg", "Wu", "Wd"))
    Wr = torch.from_numpy(inp["Wr"]).to(DEV)
    buf.run_block_fwd_bwd(x, Wr, dout, Wg, Wu, Wd)
    torch.cuda.synchronize()
    dx_block = H.bf16_from_dev(buf.dx)
    inp2 = dict(inp)
    inp2["logits"] = buf.logits.cpu().numpy()
    ref = O.layer_fwd_bwd(inp2, cfg.k, 0, cfg.E, cfg.renormalize)
    assert np.array_equal(buf.topk_idx.cpu().numpy(), ref["topk_idx"])
    np.testing.assert_allclose(inp2["logits"], O.router_logits(O.decode_bf16(inp["x"]), inp["Wr"]), rtol=0, atol=2e-5)
    rdl = O.route_bwd(inp2["logits"], ref["topk_idx"], ref["dgate"], cfg.renormalize)
    rdWr, rdx = O.router_bwd(O.decode_bf16(inp["x"]), inp["Wr"], rdl)
    H.assert_close(buf.dlogits.cpu().numpy().astype(np.float64), rdl, "dlogits")
    H.assert_close(buf.dWr.cpu().numpy().astype(np.float64), rdWr, "dWr")
    H.assert_close(dx_block, ref["dx"] + rdx, "dx (expert path + router path)")
    H.assert_close(H.bf16_from_dev(buf.out), ref["out"], "out")
    # the router's share is really in dx: the expert path alone leaves something else
    buf.run_fwd_bwd(x, buf.logits, dout, Wg, Wu, Wd)
    torch.cuda.synchronize()
    assert np.abs(dx_block - H.bf16_from_dev(buf.dx)).max() > 0


def test_layer_without_local_rows():
    """No token chooses a local expert: every offset is 0, no grouped row exists, the layer
    output and every gradient are exactly zero (and written: the buffers start as NaN)."""
    cfg = W.MoEConfig("custom", T=192, d=128, E=8, k=2, f=64, e_begin=6, e_count=2, seed=3)
    inp = W.make_inputs(cfg)
    inp["logits"][:, 6:] = -50.0          # experts 6 and 7 are never among the top 2
    res = H.run_layer(cfg, inp)
    ref = O.layer_fwd_bwd(inp, cfg.k, cfg.e_begin, cfg.n_local, cfg.renormalize)
    assert int(ref["expert_offsets"][-1]) == 0
    assert np.array_equal(res["expert_offsets"], np.zeros(3, dtype=np.int32))
    assert np.array_equal(res["topk_idx"], ref["topk_idx"])
    assert np.all(res["slot_row"] == -1)
    for n in ("out", "dx", "dgate", "dWg", "dWu", "dWd"):
        assert np.all(res[n] == 0.0), n


def test_layer_single_token():
    """T = 1: one token, k rows, every tile almost empty."""
    cfg = W.MoEConfig("custom", T=1, d=64, E=4, k=2, f=64, seed=9)
    inp = W.make_inputs(cfg)
    res = H.run_layer(cfg, inp)
    ref = O.layer_fwd_bwd(inp, cfg.k, cfg.e_begin, cfg.n_local, cfg.renormalize)
    H.compare_layer(res, ref, cfg.n_local)


def test_argument_checks():
    t = torch.zeros(64, 64, dtype=torch.float32, device=DEV)
    idx = torch.zeros(64, 2, dtype=torch.int32, device=DEV)
    w = torch.zeros(64, 2, dtype=torch.float32, device=DEV)
    lib = B.load()
    assert lib.moe_route(None, 64, 64, 2, 1, B._p(idx), B._p(w), None) == -1
    assert lib.moe_route(B._p(t), 64, 64, 65, 1, B._p(idx), B._p(w), None) == -1
    assert lib.moe_route(B._p(t), 64, 1000, 2, 1, B._p(idx), B._p(w), None) == -1
    assert lib.moe_route(t.data_ptr() + 4, 64, 64, 2, 1, B._p(idx), B._p(w), None) == -1
    x = torch.zeros(64, 64, dtype=torch.bfloat16, device=DEV)
    assert lib.moe_permute(B._p(x), B._p(idx), 64, 64, 8, 2, 0, 8, B._p(idx), B._p(idx), B._p(idx), B._p(x),
                           B._p(x), 0, None) == -2
    assert lib.moe_grouped_gemm_fwd(B._p(x), B._p(idx), B._p(x), B._p(x), B._p(x), 1, 64, 60, 64,
                                    B._p(x), B._p(x), B._p(x), B._p(x), None) == -1
    # gathered products: x, T and row_token are required
    assert lib.moe_grouped_gemm_fwd_gather(None, 64, B._p(idx), B._p(idx), B._p(x), B._p(x), B._p(x), 1, 64, 64, 64,
                                           B._p(x), B._p(x), B._p(x), B._p(x), None) == -1
    assert lib.moe_grouped_gemm_fwd_gather(B._p(x), 0, B._p(idx), B._p(idx), B._p(x), B._p(x), B._p(x), 1, 64, 64, 64,
                                           B._p(x), B._p(x), B._p(x), B._p(x), None) == -1
    assert lib.moe_grouped_gemm_fwd_gather(B._p(x), 64, None, B._p(idx), B._p(x), B._p(x), B._p(x), 1, 64, 64, 64,
                                           B._p(x), B._p(x), B._p(x), B._p(x), None) == -1
    # folded gate weights: the row weights are required, the workspace must hold the strips' partial sums too
    rw = torch.zeros(128, dtype=torch.float32, device=DEV)
    rt = torch.zeros(128, dtype=torch.int32, device=DEV)
    assert lib.moe_grouped_gemm_fwd_folded(B._p(x), 64, B._p(rt), None, B._p(idx), B._p(x), B._p(x), B._p(x), 1, 64, 64,
                                           64, B._p(x), B._p(x), B._p(x), B._p(x), None) == -1
    assert lib.moe_permute_gate(B._p(idx), None, 64, 8, 2, 0, 8, B._p(idx), B._p(rt), B._p(idx), B._p(rw), B._p(x),
                                1 << 20, None) == -1
    small = lib.moe_grouped_gemm_bwd_workspace_bytes(64, 64)
    assert lib.moe_grouped_gemm_bwd_folded_workspace_bytes(64, 64) > small
    big = torch.zeros(1 << 16, dtype=torch.uint8, device=DEV)
    assert lib.moe_grouped_gemm_bwd_folded(B._p(x), B._p(x), 64, 2, B._p(rt), B._p(rw), B._p(idx), B._p(x), B._p(x),
                                           B._p(x), B._p(idx), B._p(x), B._p(x), B._p(x), 1, 64, 64, 64, B._p(x),
                                           B._p(x), B._p(x), B._p(x), B._p(w), B._p(big), small, None) == -2
    assert lib.moe_grouped_gemm_bwd_folded(B._p(x), B._p(x), 64, 2, B._p(rt), None, B._p(idx), B._p(x), B._p(x),
                                           B._p(x), B._p(idx), B._p(x), B._p(x), B._p(x), 1, 64, 64, 64, B._p(x),
                                           B._p(x), B._p(x), B._p(x), B._p(w), B._p(big), 1 << 16, None) == -1
    # router entry points: d must be a multiple of 16, the workspace large enough, pointers aligned
    Wr = torch.zeros(8, 64, dtype=torch.float32, device=DEV)
    lg = torch.zeros(64, 8, dtype=torch.float32, device=DEV)
    assert lib.moe_router_fwd(B._p(x), B._p(Wr), 64, 40, 8, B._p(lg), None) == -1
    assert lib.moe_router_fwd(B._p(x), B._p(Wr), 0, 64, 8, B._p(lg), None) == -1
    assert lib.moe_router_fwd(B._p(x), Wr.data_ptr() + 4, 64, 64, 8, B._p(lg), None) == -1
    assert lib.moe_route_bwd(B._p(lg), B._p(idx), B._p(w), 64, 8, 9, 1, B._p(lg), None) == -1
    need = lib.moe_router_bwd_workspace_bytes(64, 64, 8)
    assert need == 1 * 8 * 64 * 4
    ws = torch.zeros(need, dtype=torch.uint8, device=DEV)
    assert lib.moe_router_bwd(B._p(x), B._p(Wr), B._p(lg), 64, 64, 8, B._p(x), B._p(Wr), B._p(ws), need - 1, None) == -2
    assert lib.moe_router_bwd(B._p(x), B._p(Wr), B._p(lg), 64, 64, 8, B._p(x), B._p(Wr), None, need, None) == -1
    torch.cuda.synchronize()


@pytest.mark.parametrize("fold", [False, True])
def test_graph_replay_matches_eager(fold):
    """The whole step recorded into a HIP graph: every replay, with eager work and
    synchronisations in between, leaves exactly the bits the eager step leaves."""
    cfg = W.MoEConfig("custom", T=700, d=256, E=16, k=4, f=128, seed=11)
    inp = W.make_inputs(cfg)
    x, dout = H.bf16_to_dev(inp["x"]), H.bf16_to_dev(inp["dout"])
    Wg, Wu, Wd = (H.bf16_to_dev(inp[n]) for n in ("Wg", "Wu", "Wd"))
    logits = torch.from_numpy(inp["logits"]).to(DEV)
    ref = B.MoELayerBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, fold=fold)
    ref.run_fwd_bwd(x, logits, dout, Wg, Wu, Wd)
    torch.cuda.synchronize()
    want = {n: t.clone() for n, t in ref.results().items()}
    buf = B.MoELayerBuffers(cfg.T, cfg.d, cfg.E, cfg.k, cfg.f, fold=fold)
    graph = buf.capture_fwd_bwd(x, logits, dout, Wg, Wu, Wd)
    for rep in range(3):
        print(f"graph replay {rep}", flush=True)
        for t in buf.results().values():
            t.fill_(1)                      # eager work between replays; stale results cannot pass
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for n, t in buf.results().items():
            R = int(want["expert_offsets"][-1])
            if n in ("xp", "g", "u", "h", "yp", "dyp", "dxp", "hw", "ypw", "row_weight"):
                assert torch.equal(t[:R], want[n][:R]), n
            elif n == "row_token":
                assert torch.equal(t[:R], want[n][:R]), n
            else:
                assert torch.equal(t, want[n]), n
