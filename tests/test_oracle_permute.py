"""Pins for oracle.permute / permute_bwd / combine identities (Algorithm 1, Stages 2-3, 5)."""
import os

import numpy as np
import pytest

from oracle import moe_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "permute_T4_N4_K2.txt")


def random_topk(rng, T, E, k):
    return np.stack([rng.permutation(E)[:k] for _ in range(T)]).astype(np.int32)


def brute_permute(topk_idx, e_begin, e_count):
    """Expert by expert, token by token, slot by slot."""
    T, k = topk_idx.shape
    offsets, row_token = [0], []
    slot_row = [[-1] * k for _ in range(T)]
    for e in range(e_begin, e_begin + e_count):
        for t in range(T):
            for i in range(k):
                if topk_idx[t, i] == e:
                    slot_row[t][i] = len(row_token)
                    row_token.append(t)
        offsets.append(len(row_token))
    return np.array(offsets), np.array(row_token), np.array(slot_row)


def blockwise_index_generation(indices, n_start, NR, TBS=8):
    """The paper's two-kernel scheme (Algorithm 1, Stages 2 and 3), written out
    from its description: token blocks of TBS tokens each own a column of a
    [local expert, block] count table; one prefix sum over that table in
    expert-major order gives every (expert, block) its first row; a second
    sweep hands out rows inside each (expert, block) in token order.  A CSR
    over tokens (cum_expert_counts) addresses each token's local picks.
    Readings: the block's token is computed before it is used; the count table
    is indexed by block id (it has NR*TH entries); n_end is inclusive;
    '[1:] = PrefixSum' is the inclusive scan stored from position 1.
    """
    T, K = indices.shape
    assert T % TBS == 0
    TH = T // TBS
    n_end = n_start + NR - 1
    partial = np.zeros(NR * TH, dtype=np.int64)
    expert_counts = np.zeros(T, dtype=np.int64)
    for tid in range(TH):
        for i in range(TBS):
            t = tid * TBS + i
            for k in range(K):
                n = indices[t, k]
                if n_start <= n <= n_end:
                    partial[(n - n_start) * TH + tid] += 1
                    expert_counts[t] += 1
    partial_cum = np.zeros(NR * TH + 1, dtype=np.int64)
    partial_cum[1:] = np.cumsum(partial)
    cum_expert = np.zeros(T + 1, dtype=np.int64)
    cum_expert[1:] = np.cumsum(expert_counts)
    cum_token = np.array([partial_cum[n * TH] for n in range(NR + 1)])
    RT = cum_token[-1]
    sel = np.zeros(RT, dtype=np.int64)
    inp = np.zeros(RT, dtype=np.int64)
    outp = np.zeros(RT, dtype=np.int64)
    counter = np.zeros((NR, TH), dtype=np.int64)
    for tid in range(TH):
        for i in range(TBS):
            t = tid * TBS + i
            o = cum_expert[t]
            for k in range(K):
                n = indices[t, k]
                if n_start <= n <= n_end:
                    ln = n - n_start
                    row = partial_cum[ln * TH + tid] + counter[ln, tid]
                    inp[row] = t
                    outp[o] = row
                    sel[o] = k
                    counter[ln, tid] += 1
                    o += 1
    return cum_token, cum_expert, inp, outp, sel


def _parse_rows(tokens):
    rows, cur = [], []
    for tok in tokens:
        if tok == "|":
            rows.append(cur)
            cur = []
        else:
            cur.append(int(tok))
    rows.append(cur)
    return np.array(rows)


def test_hand_worked_example():
    entries = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        p = line.split()
        if p[0] == "indices":
            entries["indices"] = _parse_rows(p[1:])
        else:
            name_end = 2 if p[0] == "ep1" else 3
            entries[" ".join(p[:name_end])] = p[name_end:]
    idx = entries["indices"].astype(np.int32)
    x = np.arange(4 * 3, dtype=np.float64).reshape(4, 3)
    cases = [("ep1", 0, 4), ("ep2 rank0", 0, 2), ("ep2 rank1", 2, 2)]
    for tag, eb, ec in cases:
        off, rt, sr, xp = O.permute(x, idx, eb, ec)
        assert off.tolist() == [int(v) for v in entries[f"{tag} expert_offsets"]]
        assert rt.tolist() == [int(v) for v in entries[f"{tag} row_token"]]
        assert np.array_equal(sr, _parse_rows(entries[f"{tag} slot_row"]))
        assert np.array_equal(xp, x[rt])


@pytest.mark.parametrize("T,E,k", [(16, 4, 2), (64, 8, 2), (40, 64, 8), (24, 12, 5)])
@pytest.mark.parametrize("EP", [1, 2, 4])
def test_permute_matches_brute_force_and_blockwise_scheme(T, E, k, EP):
    rng = np.random.default_rng(T + E + k + EP)
    idx = random_topk(rng, T, E, k)
    x = rng.standard_normal((T, 5))
    NR = E // EP
    for r in range(EP):
        off, rt, sr, xp = O.permute(x, idx, r * NR, NR)
        boff, brt, bsr = brute_permute(idx, r * NR, NR)
        assert np.array_equal(off, boff) and np.array_equal(rt, brt) and np.array_equal(sr, bsr)
        cum_token, cum_expert, inp, outp, sel = blockwise_index_generation(idx, r * NR, NR)
        assert np.array_equal(cum_token, off)
        assert np.array_equal(inp, rt)
        # CSR (cum_expert_counts, selected_expert_indices, output_indices) <-> dense slot_row
        for t in range(T):
            local = [(i, sr[t, i]) for i in range(k) if sr[t, i] >= 0]
            a, b = cum_expert[t], cum_expert[t + 1]
            assert [(int(sel[j]), int(outp[j])) for j in range(a, b)] == [(i, int(row)) for i, row in local]
        assert np.array_equal(xp, x[inp])


def test_permute_invariants_and_empty_experts():
    rng = np.random.default_rng(5)
    T, E, k = 300, 16, 4
    idx = random_topk(rng, T, E - 3, k)          # experts 13,14,15 never chosen
    idx[idx == 2] = 15                            # expert 2 empty, 15 used
    x = rng.standard_normal((T, 3))
    off, rt, sr, xp = O.permute(x, idx, 0, E)
    counts = np.diff(off)
    assert off[0] == 0 and np.all(counts >= 0) and off[-1] == T * k       # counts sum to T*k
    assert counts[2] == 0 and counts[13] == 0 and counts[14] == 0 and counts[15] > 0
    assert np.array_equal(np.sort(sr.reshape(-1)), np.arange(T * k))      # bijection
    assert np.array_equal(rt[sr], np.repeat(np.arange(T)[:, None], k, 1))  # row_token[slot_row[t,i]] = t
    for e in range(E):
        seg = rt[off[e]:off[e + 1]]
        assert np.all(np.diff(seg) > 0)                                   # token order inside an expert
        assert np.all(idx[seg] == e, axis=None) or np.all((idx[seg] == e).any(1))
    # slot order does not matter for the grouping: reverse every token's slots
    off2, rt2, sr2, _ = O.permute(x, idx[:, ::-1], 0, E)
    assert np.array_equal(off2, off) and np.array_equal(rt2, rt) and np.array_equal(sr2[:, ::-1], sr)


@pytest.mark.parametrize("k", [1, 2, 4, 8])
def test_permute_then_unpermute_is_identity(k):
    rng = np.random.default_rng(k)
    T, E, d = 64, 8, 16
    idx = random_topk(rng, T, E, k)
    # short mantissas (bf16-representable values) keep every partial sum exact
    x = O.decode_bf16((rng.standard_normal((T, d)).astype(np.float32).view(np.uint32) >> 16).astype(np.uint16))
    off, rt, sr, xp = O.permute(x, idx, 0, E)
    w = np.full((T, k), 1.0 / k)
    assert np.array_equal(O.combine_fwd(xp, sr, w), x)          # power-of-two scaling is exact
    assert np.array_equal(O.permute_bwd(xp, sr), k * x)


def test_permute_bwd_is_the_transpose_of_the_gather():
    """<permute(x), y> == <x, permute_bwd(y)> for the linear map x -> xp."""
    rng = np.random.default_rng(11)
    T, E, k, d = 50, 6, 3, 7
    idx = random_topk(rng, T, E, k)
    x = rng.standard_normal((T, d))
    for eb, ec in [(0, E), (2, 3)]:
        off, rt, sr, xp = O.permute(x, idx, eb, ec)
        y = rng.standard_normal(xp.shape)
        np.testing.assert_allclose((xp * y).sum(), (x * O.permute_bwd(y, sr)).sum(), rtol=1e-12)
