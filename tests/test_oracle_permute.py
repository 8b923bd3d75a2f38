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
    """Second, independent definition of the index structures, after the scheme of Algorithm 1,
    Stages 2 and 3, as the text describes it (not its listing): tokens are cut into blocks of TBS;
    a [local expert, block] table counts the picks; ONE running sum over that table, read expert by
    expert, gives every (expert, block) cell its first grouped row; inside a cell the rows go out in
    token order.  A CSR over tokens addresses each token's local picks in slot order.
    Readings taken: the local range is [n_start, n_start + NR) (the paper's n_end is inclusive); the
    count table has one column per block; the stored prefix sums start with a zero.
    Built here from whole-array operations (histogram, cumulative sum, rank inside a cell).
    """
    T, K = indices.shape
    assert T % TBS == 0
    blocks = T // TBS
    tok, slot = np.divmod(np.arange(T * K), K)               # flat pair p = t*K + slot
    local_e = indices.reshape(-1).astype(np.int64) - n_start
    keep = (local_e >= 0) & (local_e < NR)
    tok, slot, local_e = tok[keep], slot[keep], local_e[keep]      # local picks, in (token, slot) order
    cell = local_e * blocks + tok // TBS                           # expert-major cell id
    table = np.bincount(cell, minlength=NR * blocks)               # Stage 2: counts per (expert, block)
    first_row = np.concatenate(([0], np.cumsum(table)))            # one prefix sum, expert-major
    cum_token = first_row[np.arange(NR + 1) * blocks]              # first row of every expert (+ total)
    # Stage 3: rank of each pick among the earlier picks of its own cell (picks are in token order):
    # a running count per cell, read off at each pick's own cell.
    onehot = np.zeros((len(cell), NR * blocks), dtype=np.int64)
    onehot[np.arange(len(cell)), cell] = 1
    rank = (np.cumsum(onehot, axis=0) - onehot)[np.arange(len(cell)), cell]
    start_of_cell = first_row[:-1]
    row = start_of_cell[cell] + rank
    inp = np.empty(len(cell), dtype=np.int64)
    inp[row] = tok                                                  # input_indices
    per_token = np.bincount(tok, minlength=T)
    cum_expert = np.concatenate(([0], np.cumsum(per_token)))        # CSR row pointers over tokens
    return cum_token, cum_expert, inp, row, slot                   # picks are stored in CSR order already


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
