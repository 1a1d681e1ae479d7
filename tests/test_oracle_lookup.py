"""Pins for the oracle's lookup and tower-major layout (CPU only).

None of these re-type the oracle's loops: they are hand-computed numbers,
closed forms, a library routine on the special case it covers, and invariants
the paper states (Sec. 3.1: the tower transform moves data and leaves the
computation unchanged).
"""
import os

import numpy as np
import pytest
import torch

import oracle
import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _int_table(rows, D):
    r = np.arange(rows, dtype=np.float32)[:, None]
    c = np.arange(D, dtype=np.float32)[None, :]
    return 100 * r + c


def test_hand_computed_bags():
    # two tables, 5 rows, D = 4, W[r][c] = 100 r + c (table 1: plus 1000); B = 3.
    t0 = _int_table(5, 4)
    t1 = _int_table(5, 4) + 1000
    # bags in feature-major order:
    # (f0,b0) = [1, 3]   (f0,b1) = []      (f0,b2) = [4, 4, 0]
    # (f1,b0) = [2]      (f1,b1) = [0, 1, 2, 3, 4]   (f1,b2) = []
    indices = [1, 3, 4, 4, 0, 2, 0, 1, 2, 3, 4]
    offsets = [0, 2, 2, 5, 6, 11, 11]
    out = oracle.lookup_global([t0, t1], "f32", [4, 4], indices, offsets, 3)
    expect = np.array([
        # f0: rows 1+3 = 400 + 2c                    f1: row 2 = 1200 + c
        [400, 402, 404, 406, 1200, 1201, 1202, 1203],
        # f0: empty                                  f1: rows 0..4 = 5*1000 + 1000 + 5c
        [0, 0, 0, 0, 6000, 6005, 6010, 6015],
        # f0: rows 4+4+0 = 800 + 3c                  f1: empty
        [800, 803, 806, 809, 0, 0, 0, 0]], dtype=np.float64)
    assert np.array_equal(out, expect)
    # the same through the towered entry with one tower per table, swapped order
    tw = oracle.lookup_towered([t0, t1], "f32", [4, 4], [1, 0], indices, offsets, 3)
    assert np.array_equal(tw[0], expect[:, 4:])      # tower 0 owns table 1
    assert np.array_equal(tw[1], expect[:, :4])


@pytest.mark.parametrize("dtype", ["f32", "f16", "bf16"])
def test_identity_table_gives_histogram(dtype):
    D = 16
    tab = wl.encode(np.eye(D, dtype=np.float32), dtype)
    rng = np.random.default_rng(5)
    B = 40
    lens = rng.integers(0, 9, size=B)
    offsets = np.concatenate([[0], np.cumsum(lens)])
    indices = rng.integers(0, D, size=offsets[-1])
    out = oracle.lookup_global([tab], dtype, [D], indices, offsets, B)
    for b in range(B):
        hist = np.bincount(indices[offsets[b]:offsets[b + 1]], minlength=D)
        assert np.array_equal(out[b], hist.astype(np.float64))


def test_length_one_bags_are_a_row_gather():
    rng = np.random.default_rng(6)
    tab = rng.standard_normal((50, 8)).astype(np.float32)
    B = 33
    indices = rng.integers(0, 50, size=B)
    offsets = np.arange(B + 1)
    out = oracle.lookup_global([tab], "f32", [8], indices, offsets, B)
    assert np.array_equal(out, tab[indices].astype(np.float64))


def test_against_torch_embedding_bag():
    rng = np.random.default_rng(7)
    F, B, rows, D = 3, 29, 200, 24
    tabs = [rng.standard_normal((rows, D)) for _ in range(F)]          # float64 values
    tabs32 = [t.astype(np.float32) for t in tabs]
    lens = rng.integers(0, 12, size=F * B)
    offsets = np.concatenate([[0], np.cumsum(lens)])
    indices = rng.integers(0, rows, size=offsets[-1])
    out = oracle.lookup_global(tabs32, "f32", [D] * F, indices, offsets, B)
    for f in range(F):
        lo, hi = offsets[f * B], offsets[(f + 1) * B]
        ref = torch.nn.functional.embedding_bag(
            torch.from_numpy(indices[lo:hi]), torch.from_numpy(tabs32[f].astype(np.float64)),
            torch.from_numpy(offsets[f * B:(f + 1) * B] - lo), mode="sum").numpy()
        np.testing.assert_allclose(out[:, f * D:(f + 1) * D], ref, rtol=1e-13, atol=1e-13)


def test_sixteen_bit_tables_decode_exactly():
    rng = np.random.default_rng(8)
    x = (rng.standard_normal((64, 8)) * 0.01).astype(np.float32)
    for dtype, tt in (("f16", torch.float16), ("bf16", torch.bfloat16)):
        st = wl.encode(x, dtype)
        ref = torch.from_numpy(x).to(tt).to(torch.float64).numpy()
        assert np.array_equal(oracle.decode(st, dtype), ref)
        out = oracle.lookup_global([st], dtype, [8], np.arange(64), np.arange(65), 64)
        assert np.array_equal(out, ref)


def test_linearity_in_tables():
    rng = np.random.default_rng(9)
    F, B, rows, D = 2, 17, 30, 8
    a = [rng.integers(-8, 8, size=(rows, D)).astype(np.float32) for _ in range(F)]
    c = [rng.integers(-8, 8, size=(rows, D)).astype(np.float32) for _ in range(F)]
    lens = rng.integers(0, 6, size=F * B)
    offsets = np.concatenate([[0], np.cumsum(lens)])
    indices = rng.integers(0, rows, size=offsets[-1])
    f = lambda tabs: oracle.lookup_global(tabs, "f32", [D] * F, indices, offsets, B)
    lhs = f([2 * x + 3 * y for x, y in zip(a, c)])
    assert np.array_equal(lhs, 2 * f(a) + 3 * f(c))


def test_permuting_ids_inside_a_bag_changes_nothing():
    rng = np.random.default_rng(10)
    tab = rng.integers(-50, 50, size=(40, 8)).astype(np.float32)
    B = 12
    lens = rng.integers(2, 9, size=B)
    offsets = np.concatenate([[0], np.cumsum(lens)])
    indices = rng.integers(0, 40, size=offsets[-1])
    shuffled = indices.copy()
    for b in range(B):
        seg = shuffled[offsets[b]:offsets[b + 1]]
        shuffled[offsets[b]:offsets[b + 1]] = rng.permutation(seg)
    a = oracle.lookup_global([tab], "f32", [8], indices, offsets, B)
    c = oracle.lookup_global([tab], "f32", [8], shuffled, offsets, B)
    assert np.array_equal(a, c)


def _python_layout(dims, t2t, B):
    """Ten-line reference of the tower-major layout [T][B][W_t]."""
    T = max(t2t) + 1
    width = [0] * T
    col = []
    for f, t in enumerate(t2t):
        col.append(width[t])
        width[t] += dims[f]
    base = [0]
    for t in range(T):
        base.append(base[-1] + B * width[t])
    return base, width, col


@pytest.mark.parametrize("seed", [0, 1, 2, 3])
def test_tower_concatenation_equals_untowered_lookup(seed):
    """Sec. 3.1 / Table 3: regrouping features into towers leaves every pooled
    vector unchanged, for any partition; only its place in memory moves."""
    rng = np.random.default_rng(seed)
    F, B = 9, 21
    dims = [int(d) for d in rng.choice([8, 16, 24], size=F)]
    rows = [int(r) for r in rng.integers(5, 60, size=F)]
    T = int(rng.integers(1, 5))
    t2t = list(rng.permutation(np.concatenate([np.arange(T), rng.integers(0, T, size=F - T)])))
    tabs = [rng.standard_normal((rows[f], dims[f])).astype(np.float32) for f in range(F)]
    lens = rng.integers(0, 7, size=F * B)
    offsets = np.concatenate([[0], np.cumsum(lens)])
    indices = np.concatenate([rng.integers(0, rows[f], size=offsets[(f + 1) * B] - offsets[f * B])
                              for f in range(F)])
    glob = oracle.lookup_global(tabs, "f32", dims, indices, offsets, B)
    tow = oracle.lookup_towered(tabs, "f32", dims, t2t, indices, offsets, B)
    base, width, col = _python_layout(dims, t2t, B)
    assert [t.shape for t in tow] == [(B, w) for w in width]
    gcol = np.concatenate([[0], np.cumsum(dims)])
    for f in range(F):
        piece = tow[t2t[f]][:, col[f]:col[f] + dims[f]]
        assert np.array_equal(piece, glob[:, gcol[f]:gcol[f + 1]])
    # and the workload module's own layout helper agrees with the reference
    w = wl.Workload("x", 0, rows, dims, "f32", [int(t) for t in t2t], B, "uniform", 1, 1, None,
                    wl.TM_LINEAR, [8] * T, 0, "f32", "f32", False)
    assert wl.pooled_layout(w) == (base, width, col)


def test_paper_naive_partition_layout():
    """The 8-tower strided partition the paper lists (Sec. 5.2.3) as a fixture:
    tower sizes 4,4,3,3,3,3,3,3 and `embs` of shape (B, |F|, N) per tower."""
    towers = [[int(x) for x in l.split()] for l in open(os.path.join(GOLD, "naive_partition_8_towers.txt"))
              if l.strip() and not l.startswith("#")]
    assert [len(t) for t in towers] == [4, 4, 3, 3, 3, 3, 3, 3]
    t2t = [0] * 26
    for t, fs in enumerate(towers):
        for f in fs:
            assert f % 8 == t
            t2t[f] = t
    N, B = 8, 5
    rng = np.random.default_rng(11)
    tabs = [rng.integers(-9, 9, size=(7, N)).astype(np.float32) for _ in range(26)]
    lens = rng.integers(0, 4, size=26 * B)
    offsets = np.concatenate([[0], np.cumsum(lens)])
    indices = rng.integers(0, 7, size=offsets[-1])
    tow = oracle.lookup_towered(tabs, "f32", [N] * 26, t2t, indices, offsets, B)
    glob = oracle.lookup_global(tabs, "f32", [N] * 26, indices, offsets, B).reshape(B, 26, N)
    for t, fs in enumerate(towers):
        embs = tow[t].reshape(B, len(fs), N)            # (B, |F|, N)
        assert np.array_equal(embs, glob[:, fs, :])


def test_round_to_matches_torch():
    rng = np.random.default_rng(12)
    x = np.concatenate([
        rng.standard_normal(5000) * 10.0 ** rng.integers(-45, 38, size=5000),
        [0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e39, -1e39, 1e-41, 9.2e-41, 4.6e-41],
    ]).astype(np.float32).astype(np.float64)
    ref = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got = oracle.round_to(x, "bf16")
    assert np.array_equal(got, ref)
    # a double that lies between float32 neighbours across a bf16 tie must round directly
    tie = 1.0 + 2.0 ** -8                      # exact tie between 1.0 and 1.0078125 -> even (1.0)
    assert oracle.round_to(np.array([tie, tie + 2.0 ** -40]), "bf16").tolist() == [0x3F80, 0x3F81]
    h = oracle.round_to(x, "f16")
    with np.errstate(over="ignore"):
        assert np.array_equal(h.view(np.uint16),
                              torch.from_numpy(x).to(torch.float16).view(torch.int16).numpy().view(np.uint16))
