"""SPTT's data-shuffle steps on one GPU, and a whole simulated cluster, CPU oracle.
TEST INFRASTRUCTURE ONLY.

Only tests may import this module; the product package never does, and nothing
here touches the HIP library.

The Semantic-Preserving Tower Transform (paper Sec. 3.1.1) replaces the global
embedding AlltoAll by: (a) global distribution of the sparse inputs, (b) local
lookup, (c) peer permute, (d) intra-host exchange, (e) a (features, peers) ->
(peers, features) shuffle, (f) concurrent AlltoAlls among peers.  Steps c and e
move blocks of data inside one GPU's memory; they are written here on numpy
arrays exactly as the walk-through states them, and `simulate` plays all six
steps for G virtual GPUs so that the result can be held against the plain
definition of the embedding lookup (the transform does not change the model).

Setting (the walk-through's): G GPUs, L per host, T = G / L hosts, one tower
per host; the tower's tables are placed whole on its host's GPUs; every GPU
contributes B_l samples, rank g owning samples [g B_l, (g + 1) B_l).

Reading: the walk-through sorts by the key (g % T, g // L) while it defines
peers through g % L; its example has T = L = 2 and cannot tell the two apart.
With G = 8, L = 4, T = 2 the printed key has ties and does not bring peers
together; (g % L, g // L) does, and gives the printed order (0, 2, 1, 3) for the
example.  That key is used here.

`peer_permute_ids` is step c moved in front of step b (Sec. 3.1.3): the permute acts on the
jagged sparse inputs.  `row_shard_lookups` covers the row-wise sharded variant of Sec. 3.1.3: the part
of a batch's lookups one row shard of the tables serves.

Pinned in tests/test_oracle_sptt.py against the paper's example, hand-labelled
blocks, the end-to-end simulation against the definition of the lookup, and
(row shards) a hand case and partial pools that add up to the lookup.
"""
from __future__ import annotations

from typing import List, Sequence

import numpy as np


def peers(g: int, G: int, L: int) -> List[int]:
    """Ranks g_j with g_j % L == g % L (Sec. 3.1.1), ascending."""
    return [r for r in range(G) if r % L == g % L]


def peer_order(G: int, L: int) -> List[int]:
    """All ranks sorted by the key (g % L, g // L): peers end up next to one another, ordered by
    host (Sec. 3.1.1 step c; the key as read in this module's header)."""
    if G <= 0 or L <= 0 or G % L != 0:
        raise ValueError("L must divide G")
    return sorted(range(G), key=lambda g: (g % L, g // L))


def peer_permute(x: np.ndarray, L: int) -> np.ndarray:
    """Step c.  `x` is (features, G, ...): for every local feature the blocks received from the
    G ranks, in rank order.  Returns them in peer order."""
    G = x.shape[1]
    return np.ascontiguousarray(x[:, peer_order(G, L)])


def shuffle(z: np.ndarray) -> np.ndarray:
    """Step e.  `z` is (features, peers, ...): stack as a 2-D arrangement of blocks, transpose it
    to (peers, features), flattened in that order."""
    return np.ascontiguousarray(np.swapaxes(z, 0, 1))


def simulate(pooled_of, tower_tables: Sequence[Sequence[int]], L: int, B_l: int):
    """All six steps for G = len(tower_tables) * L virtual GPUs.

    pooled_of(f, lo, hi) -> the pooled embeddings (hi - lo, N) of table f for the global samples
    [lo, hi): the lookup itself (steps a and b deliver exactly these to the GPU that owns f).
    tower_tables[t] lists tower t's tables; they are dealt to host t's GPUs round-robin.
    Returns out[g][t] = array (tables of tower t, B_l, N): what GPU g holds after step f, the
    pooled embeddings of every tower's features for g's own samples.
    """
    T = len(tower_tables)
    G = T * L
    local_tables = [[] for _ in range(G)]
    for t, fs in enumerate(tower_tables):
        for i, f in enumerate(fs):
            local_tables[t * L + i % L].append(f)
    # steps a + b: GPU r holds, per local table, the blocks of all G ranks in rank order
    held = []
    for r in range(G):
        fs = local_tables[r]
        blocks = [np.stack([pooled_of(f, g * B_l, (g + 1) * B_l) for g in range(G)]) for f in fs]
        held.append(np.stack(blocks) if fs else None)           # (F_loc, G, B_l, N)
    # step c on every GPU
    permuted = [peer_permute(h, L) if h is not None else None for h in held]
    # step d: inside host t, the GPU with local index l collects, from every GPU of the host, the
    # T blocks of its own peers (positions [l T, (l + 1) T) of the peer order), for all features
    after_d = []
    for r in range(G):
        t, l = divmod(r, L)
        parts, names = [], []
        for src in range(t * L, (t + 1) * L):
            if permuted[src] is None:
                continue
            parts.append(permuted[src][:, l * T:(l + 1) * T])
            names += local_tables[src]
        z = np.concatenate(parts, axis=0)                          # (F_t, T peers, B_l, N)
        order = np.argsort([list(tower_tables[t]).index(f) for f in names])
        after_d.append(z[order])                                   # features in the tower's order
    # step e on every GPU
    shuffled = [shuffle(z) for z in after_d]                       # (T peers, F_t, B_l, N)
    # step f: AlltoAll among peers (same local index, one per host): block p goes to the peer on
    # host p; the block received from host t holds tower t's features for the receiver's samples
    out = []
    for r in range(G):
        t, l = divmod(r, L)
        out.append([shuffled[src_host * L + l][t] for src_host in range(T)])
    return out


def peer_permute_ids(indices, offsets, features: int, G: int, L: int, B_l: int):
    """Steps b and c swapped (Sec. 3.1.3: the shuffle may act on the sparse inputs instead of
    the embeddings, whichever is smaller).  `indices` / `offsets` hold, feature-major, the bags
    of `features` local features for the samples of all G ranks in rank order (bag (f, g, b) of
    feature f, rank g, sample b is number (f G + g) B_l + b).  Returns the same jagged batch with
    every feature's G blocks of B_l bags in peer order, so that a lookup on it yields what step
    c would have made of the lookup on the input."""
    indices = np.asarray(indices)
    offsets = np.asarray(offsets, dtype=np.int64)
    order = peer_order(G, L)
    out_idx, lens = [], []
    for f in range(features):
        for g in order:
            first = (f * G + g) * B_l
            lo, hi = offsets[first], offsets[first + B_l]
            out_idx.append(indices[lo:hi])
            lens.append(np.diff(offsets[first:first + B_l + 1]))
    new_idx = np.concatenate(out_idx) if out_idx else indices[:0]
    new_off = np.concatenate([[0], np.cumsum(np.concatenate(lens))]).astype(np.int64) if lens \
        else np.zeros(1, np.int64)
    return new_idx.astype(indices.dtype), new_off


# ------------------------------------------------------------------ row-wise sharded tables

def row_shard_lookups(indices, offsets, F: int, B: int, row_begin: Sequence[int],
                      rows: Sequence[int]):
    """The lookups of a batch that fall into one row-wise shard (Sec. 3.1.3: a table too large
    for one GPU is split by rows inside its tower; every shard pools the rows it holds and step d
    becomes a ReduceScatter that adds the partial pools).

    The shard holds rows [row_begin[f], row_begin[f] + rows[f]) of table f.  Returns the jagged
    batch restricted to those rows, ids renumbered from the shard's first row: (indices, offsets)
    in the same feature-major layout, the order inside every bag kept."""
    indices = np.asarray(indices, dtype=np.int64)
    offsets = np.asarray(offsets, dtype=np.int64)
    table_of = np.repeat(np.arange(F), np.diff(offsets[::B]))
    lo = np.asarray(row_begin, dtype=np.int64)[table_of]
    hi = lo + np.asarray(rows, dtype=np.int64)[table_of]
    keep = (indices >= lo) & (indices < hi)
    kept_before = np.concatenate([[0], np.cumsum(keep)])
    return (indices - lo)[keep].astype(np.int32), kept_before[offsets]
