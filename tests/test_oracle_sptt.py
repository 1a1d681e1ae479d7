"""Pins of the SPTT shuffle oracle (oracle/sptt.py; paper Sec. 3.1.1): the paper's example, hand
cases on labelled blocks, and the whole transform on a simulated cluster against the definition
of the lookup it must not change."""
import os

import numpy as np
import pytest

from oracle import sptt

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_peer_order_of_the_papers_example():
    rows = [[int(x) for x in l.split()] for l in open(os.path.join(GOLD, "peer_order_example.txt"))
            if l.strip() and not l.startswith("#")]
    for G, L, *order in rows:
        assert sptt.peer_order(G, L) == order
    assert sptt.peer_order(4, 2) == [0, 2, 1, 3]


def test_peer_order_groups_peers_by_host():
    for G, L in ((8, 4), (8, 2), (16, 8), (6, 3), (5, 1), (4, 4)):
        T = G // L
        order = sptt.peer_order(G, L)
        assert sorted(order) == list(range(G))
        for l in range(L):
            group = order[l * T:(l + 1) * T]
            assert group == sptt.peers(l, G, L)              # one peer group, ascending host
            assert [g // L for g in group] == list(range(T))
    # the key as printed, (g % T, g // L), does not do that once T != L
    printed = sorted(range(8), key=lambda g: (g % 2, g // 4))
    assert printed[:2] != sptt.peers(0, 8, 4)
    with pytest.raises(ValueError):
        sptt.peer_order(6, 4)


def test_peer_permute_and_shuffle_on_labelled_blocks():
    # block (f, g) holds the value 10 f + g
    F, G, L = 2, 4, 2
    x = (10 * np.arange(F)[:, None] + np.arange(G)[None, :]).astype(np.float64)[:, :, None]
    y = sptt.peer_permute(x, L)
    assert y[:, :, 0].tolist() == [[0, 2, 1, 3], [10, 12, 11, 13]]
    z = (10 * np.arange(3)[:, None] + np.arange(2)[None, :]).astype(np.float64)[:, :, None]   # (features, peers)
    s = sptt.shuffle(z)
    assert s.shape == (2, 3, 1)
    assert s[:, :, 0].tolist() == [[0, 10, 20], [1, 11, 21]]
    assert s.reshape(-1).tolist() == [0, 10, 20, 1, 11, 21]      # flattened (peers x features)


@pytest.mark.parametrize("T,L,per_tower", [(2, 2, [1, 1]), (2, 2, [2, 2]), (2, 4, [5, 4]), (3, 2, [2, 3, 1]),
                                           (4, 1, [2, 2, 2, 2]), (1, 4, [6])])
def test_the_transform_keeps_the_lookup(T, L, per_tower):
    """After steps a-f every GPU holds, per tower, the pooled embeddings of that tower's features
    for its own samples: exactly what the plain lookup gives."""
    rng = np.random.default_rng(T * 10 + L)
    B_l, N = 3, 4
    G = T * L
    F = sum(per_tower)
    ids = list(rng.permutation(F))                  # towers own arbitrary table ids
    tower_tables, k = [], 0
    for n in per_tower:
        tower_tables.append([int(f) for f in ids[k:k + n]])
        k += n
    truth = rng.normal(size=(F, G * B_l, N))        # pooled embedding of table f for every global sample
    out = sptt.simulate(lambda f, lo, hi: truth[f, lo:hi], tower_tables, L, B_l)
    assert len(out) == G
    for g in range(G):
        for t in range(T):
            got = out[g][t]
            assert got.shape == (per_tower[t], B_l, N)
            for i, f in enumerate(tower_tables[t]):
                np.testing.assert_array_equal(got[i], truth[f, g * B_l:(g + 1) * B_l])


# ------------------------------------------------------------------ row-wise shards (Sec. 3.1.3)

def test_row_shard_lookups_hand_case():
    # one table, B = 3 bags: [0 5 9] [] [4 5 5 1]; the shard holds rows 4 .. 7
    idx = np.array([0, 5, 9, 4, 5, 5, 1], dtype=np.int32)
    off = np.array([0, 3, 3, 7], dtype=np.int64)
    s_idx, s_off = sptt.row_shard_lookups(idx, off, 1, 3, [4], [4])
    assert s_idx.tolist() == [1, 0, 1, 1] and s_off.tolist() == [0, 1, 1, 4]
    # a shard that holds everything changes nothing; one that holds nothing leaves empty bags
    a_idx, a_off = sptt.row_shard_lookups(idx, off, 1, 3, [0], [10])
    assert a_idx.tolist() == idx.tolist() and a_off.tolist() == off.tolist()
    n_idx, n_off = sptt.row_shard_lookups(idx, off, 1, 3, [10], [5])
    assert len(n_idx) == 0 and n_off.tolist() == [0, 0, 0, 0]


def test_partial_pools_of_the_shards_add_up_to_the_lookup():
    import oracle
    rng = np.random.default_rng(3)
    F, B, D = 3, 6, 4
    rows = [11, 7, 20]
    tables = [rng.integers(-8, 8, size=(r, D)).astype(np.float32) for r in rows]   # exact sums
    lens = rng.integers(0, 5, size=F * B)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    idx = np.concatenate([rng.integers(0, rows[f], size=int(lens[f * B:(f + 1) * B].sum()))
                          for f in range(F)]).astype(np.int32)
    t2t = [0, 1, 0]
    full = oracle.lookup_towered(tables, "f32", [D] * F, t2t, idx, off, B)
    cuts = [[0, 4, 11], [0, 7, 7], [0, 1, 20]]          # two shards per table, one of them empty
    total = [np.zeros_like(t) for t in full]
    for s in range(2):
        lo = [cuts[f][s] for f in range(F)]
        n = [cuts[f][s + 1] - cuts[f][s] for f in range(F)]
        shard_tables = [tables[f][lo[f]:lo[f] + n[f]] if n[f] else np.zeros((1, D), np.float32)
                        for f in range(F)]
        s_idx, s_off = sptt.row_shard_lookups(idx, off, F, B, lo, n)
        part = oracle.lookup_towered(shard_tables, "f32", [D] * F, t2t, s_idx, s_off, B)
        for t in range(2):
            total[t] += part[t]
    for t in range(2):
        np.testing.assert_array_equal(total[t], full[t])


def test_peer_permute_ids_hand_case():
    # one feature, G = 4 ranks, L = 2 per host, one sample per rank; bags of ranks 0..3 hold
    # [10], [20, 21], [40], [30, 31, 32]; peer order is (0, 2, 1, 3)
    idx = np.array([10, 20, 21, 40, 30, 31, 32], dtype=np.int32)
    off = np.array([0, 1, 3, 4, 7], dtype=np.int64)
    new_idx, new_off = sptt.peer_permute_ids(idx, off, 1, 4, 2, 1)
    assert new_idx.tolist() == [10, 40, 20, 21, 30, 31, 32]
    assert new_off.tolist() == [0, 1, 2, 4, 7]
    # two samples per rank, an empty bag: rank blocks [[1], [2, 3]], [[], [4]], [[5, 6], []], [[7], [8]]
    idx = np.arange(1, 9, dtype=np.int32)
    off = np.array([0, 1, 3, 3, 4, 6, 6, 7, 8], dtype=np.int64)
    new_idx, new_off = sptt.peer_permute_ids(idx, off, 1, 4, 2, 2)
    assert new_idx.tolist() == [1, 2, 3, 5, 6, 4, 7, 8]
    assert new_off.tolist() == [0, 1, 3, 5, 5, 5, 6, 7, 8]
    # two features: every feature's blocks are permuted inside the feature's own range
    idx2 = np.concatenate([idx, idx + 100]).astype(np.int32)
    off2 = np.concatenate([off, off[1:] + 8])
    new_idx2, new_off2 = sptt.peer_permute_ids(idx2, off2, 2, 4, 2, 2)
    assert new_idx2.tolist() == new_idx.tolist() + (new_idx + 100).tolist()
    assert new_off2.tolist() == new_off.tolist() + (new_off[1:] + 8).tolist()


@pytest.mark.parametrize("G,L,Bl", [(4, 2, 3), (8, 4, 2), (6, 3, 5), (2, 2, 4), (3, 1, 2)])
def test_lookup_on_permuted_ids_is_the_permuted_lookup(G, L, Bl):
    """Swapping steps b and c does not change what step c hands to step d: the pooled embeddings
    of a lookup on the permuted ids are, block for block, the peer permute of the pooled
    embeddings of the lookup on the ids as they arrived."""
    import oracle
    rng = np.random.default_rng(G * 100 + L)
    F, N, rows = 3, 4, 50
    B = G * Bl
    lens = rng.integers(0, 5, size=F * B)
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    idx = rng.integers(0, rows, size=int(off[-1])).astype(np.int32)
    tables = [rng.standard_normal((rows, N)).astype(np.float32) for _ in range(F)]
    t2t = [0] * F

    def pooled(i, o):                    # (F, G, Bl, N): tower-major [B][F N] -> per feature blocks
        out = oracle.lookup_towered(tables, "f32", [N] * F, t2t, i, o, B)[0]
        return np.ascontiguousarray(out.reshape(B, F, N).transpose(1, 0, 2)).reshape(F, G, Bl, N)

    new_idx, new_off = sptt.peer_permute_ids(idx, off, F, G, L, Bl)
    assert np.array_equal(np.sort(new_idx), np.sort(idx)) and new_off[-1] == off[-1]
    assert np.array_equal(pooled(new_idx, new_off), sptt.peer_permute(pooled(idx, off), L))
