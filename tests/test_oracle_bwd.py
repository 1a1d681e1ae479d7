"""Pins for the oracle's backward (CPU only): library sort / unique, brute-force
rank on tiny inputs, gradient-sum conservation, finite differences of the
(linear) lookup, textbook Adagrad at D = 1, a hand-computed update."""
import numpy as np
import pytest
import torch

import oracle


def _batch(rng, F, B, rows, maxlen=6):
    lens = rng.integers(0, maxlen + 1, size=F * B)
    offsets = np.concatenate([[0], np.cumsum(lens)])
    indices = np.concatenate([rng.integers(0, rows[f], size=offsets[(f + 1) * B] - offsets[f * B])
                              for f in range(F)]).astype(np.int32)
    return indices, offsets


def _table_of_pos(F, B, offsets):
    t = np.empty(offsets[-1], dtype=np.int64)
    for f in range(F):
        t[offsets[f * B]:offsets[(f + 1) * B]] = f
    return t


def test_sort_against_numpy_stable_argsort_and_unique():
    rng = np.random.default_rng(0)
    F, B, rows = 5, 40, [7, 3, 50, 11, 2]
    indices, offsets = _batch(rng, F, B, rows)
    st, sr, sp = oracle.sort_keys(F, B, indices, offsets)
    tab = _table_of_pos(F, B, offsets)
    key = tab * (1 << 32) + indices
    order = np.argsort(key, kind="stable")
    assert np.array_equal(sp, order)
    assert np.array_equal(st, tab[order]) and np.array_equal(sr, indices[order])
    ut, ur, so = oracle.unique(st, sr)
    uk, first, counts = np.unique(key, return_index=True, return_counts=True)
    assert np.array_equal(ut * (1 << 32) + ur, uk)
    assert np.array_equal(so, np.concatenate([[0], np.cumsum(counts)]))
    assert np.array_equal(np.diff(so), counts)


def test_sort_brute_force_rank_tiny():
    rng = np.random.default_rng(1)
    F, B, rows = 2, 6, [4, 3]
    indices, offsets = _batch(rng, F, B, rows, maxlen=5)
    n = len(indices)
    assert 8 <= n <= 64
    st, sr, sp = oracle.sort_keys(F, B, indices, offsets)
    tab = _table_of_pos(F, B, offsets)
    for j in range(n):                                   # O(n^2): rank = #smaller + #equal before
        rank = sum((tab[i], indices[i]) < (tab[j], indices[j]) or
                   ((tab[i], indices[i]) == (tab[j], indices[j]) and i < j) for i in range(n))
        assert sp[rank] == j


def test_empty_batch():
    F, B = 3, 4
    st, sr, sp = oracle.sort_keys(F, B, np.zeros(0, np.int32), np.zeros(F * B + 1, np.int64))
    assert len(st) == 0
    ut, ur, so = oracle.unique(st, sr)
    assert len(ut) == 0 and so.tolist() == [0]


def _setup(seed, F=4, B=25, T=2):
    rng = np.random.default_rng(seed)
    dims = [int(d) for d in rng.choice([4, 8], size=F)]
    rows = [int(r) for r in rng.integers(3, 15, size=F)]
    t2t = [f % T for f in range(F)]
    indices, offsets = _batch(rng, F, B, rows)
    widths = [sum(dims[f] for f in range(F) if t2t[f] == t) for t in range(T)]
    grad = rng.standard_normal(B * sum(widths)).astype(np.float32)
    return rng, dims, rows, t2t, indices, offsets, widths, grad


def _grad_slice(grad, dims, t2t, widths, B, f, b):
    T = len(widths)
    base = np.concatenate([[0], np.cumsum([B * w for w in widths])])
    col = sum(dims[g] for g in range(f) if t2t[g] == t2t[f])
    s = base[t2t[f]] + b * widths[t2t[f]] + col
    return grad[s:s + dims[f]].astype(np.float64)


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_gradient_sum_conservation(seed):
    """Summed over a table's touched rows, the row gradients equal the sum over
    bags of (bag length) x (that bag's output gradient)."""
    _, dims, rows, t2t, indices, offsets, widths, grad = _setup(seed)
    F, B = len(dims), 25
    kt, kr, G = oracle.bwd_accumulate(dims, t2t, indices, offsets, B, grad)
    assert np.all(np.diff(kt * (1 << 32) + kr) > 0)            # ascending, distinct
    for f in range(F):
        lhs = G[kt == f][:, :dims[f]].sum(axis=0)
        rhs = np.zeros(dims[f])
        for b in range(B):
            ln = offsets[f * B + b + 1] - offsets[f * B + b]
            rhs += ln * _grad_slice(grad, dims, t2t, widths, B, f, b)
        np.testing.assert_allclose(lhs, rhs, rtol=1e-12, atol=1e-12)
        assert (G[kt == f][:, dims[f]:] == 0).all()
    # the set of touched keys is the set numpy.unique finds
    tab = _table_of_pos(F, B, offsets)
    assert np.array_equal(kt * (1 << 32) + kr, np.unique(tab * (1 << 32) + indices))


def test_row_gradient_is_the_derivative_of_the_lookup():
    """L = <towered lookup output, grad> is linear in every table entry, so a
    finite difference is exact up to rounding: dL/dW_f[r][d] = G[(f, r)][d]."""
    rng, dims, rows, t2t, indices, offsets, widths, grad = _setup(5)
    F, B = len(dims), 25
    tabs = [rng.standard_normal((rows[f], dims[f])) for f in range(F)]

    def loss(ts):
        tow = oracle.lookup_towered([t.astype(np.float32) for t in ts], "f32", dims, t2t,
                                    indices, offsets, B)
        flat = np.concatenate([t.reshape(-1) for t in tow])
        return float(flat @ grad.astype(np.float64))

    tabs = [np.round(t * 64) / 64 for t in tabs]                # exact in float32
    kt, kr, G = oracle.bwd_accumulate(dims, t2t, indices, offsets, B, grad)
    lookup = {(int(a), int(b)): g for a, b, g in zip(kt, kr, G)}
    base = loss(tabs)
    for f in range(F):
        for r in range(rows[f]):
            for d in (0, dims[f] - 1):
                pert = [t.copy() for t in tabs]
                pert[f][r, d] += 0.5
                fd = (loss(pert) - base) / 0.5
                expect = lookup.get((f, r), np.zeros(8))[d]
                assert abs(fd - expect) < 1e-9 * max(1.0, abs(expect))


def test_single_occurrence_row_gets_that_bags_gradient():
    dims, t2t, B = [4, 4], [0, 1], 2
    indices = np.array([3, 1, 2, 0], dtype=np.int32)            # every bag has one id
    offsets = np.arange(5)
    grad = np.arange(16, dtype=np.float32)                      # tower0: [b0: 0..3, b1: 4..7], tower1: 8..15
    kt, kr, G = oracle.bwd_accumulate(dims, t2t, indices, offsets, B, grad)
    assert list(zip(kt, kr)) == [(0, 1), (0, 3), (1, 0), (1, 2)]
    assert G.tolist() == [[4, 5, 6, 7], [0, 1, 2, 3], [12, 13, 14, 15], [8, 9, 10, 11]]


def test_repeated_id_in_one_bag_counts_twice():
    kt, kr, G = oracle.bwd_accumulate([2], [0], np.array([5, 5, 5, 1], np.int32), np.array([0, 3, 4]),
                                      2, np.array([1.0, 2.0, 10.0, 20.0], np.float32))
    assert list(zip(kt, kr)) == [(0, 1), (0, 5)]
    assert G.tolist() == [[10, 20], [3, 6]]


def test_adagrad_matches_textbook_at_d1():
    """With D = 1 the rowwise rule is plain Adagrad (eps outside the root), so
    torch.optim.Adagrad on a vector of scalars must agree over several steps."""
    rng = np.random.default_rng(3)
    n, lr, eps = 12, 0.05, 1e-8
    w0 = rng.standard_normal(n)
    p = torch.nn.Parameter(torch.from_numpy(w0.copy()))
    opt = torch.optim.Adagrad([p], lr=lr, eps=eps, initial_accumulator_value=0.0)
    w, s = w0.reshape(n, 1).copy(), np.zeros(n)
    for step in range(4):
        g = rng.standard_normal(n)
        p.grad = torch.from_numpy(g.copy())
        opt.step()
        w, s = oracle.rowwise_adagrad(w, s, g.reshape(n, 1), np.ones(n, np.int32), lr, eps)
        np.testing.assert_allclose(w[:, 0], p.detach().numpy(), rtol=1e-12, atol=1e-14)


def test_adagrad_hand_computed_rows():
    # row 0: D = 4, G = (1, -1, 2, 0): mean square = 6/4 = 1.5; state 0.1 -> 1.6
    # row 1: D = 2 (padded to 4), G = (3, 4): mean square = 12.5; state 0 -> 12.5
    G = np.array([[1.0, -1.0, 2.0, 0.0], [3.0, 4.0, 0.0, 0.0]])
    w = np.array([[1.0, 1.0, 1.0, 1.0], [0.5, -0.5, 7.0, 7.0]])
    w2, s2 = oracle.rowwise_adagrad(w, np.array([0.1, 0.0]), G, np.array([4, 2], np.int32), 0.1, 0.0)
    assert s2.tolist() == [1.6, 12.5]
    r0 = 0.1 / np.sqrt(1.6)
    np.testing.assert_allclose(w2[0], [1 - r0, 1 + r0, 1 - 2 * r0, 1.0], rtol=1e-15)
    r1 = 0.1 / np.sqrt(12.5)
    np.testing.assert_allclose(w2[1], [0.5 - 3 * r1, -0.5 - 4 * r1, 7.0, 7.0], rtol=1e-15)
    # lr = 0 leaves rows alone but still advances the state
    w3, s3 = oracle.rowwise_adagrad(w, np.array([0.1, 0.0]), G, np.array([4, 2], np.int32), 0.0, 1e-8)
    assert np.array_equal(w3, w) and s3.tolist() == [1.6, 12.5]


def test_bwd_update_touches_only_activated_rows():
    rng, dims, rows, t2t, indices, offsets, widths, grad = _setup(7)
    F, B = len(dims), 25
    tabs = [rng.standard_normal((rows[f], dims[f])).astype(np.float32) for f in range(F)]
    states = [np.abs(rng.standard_normal(rows[f])).astype(np.float32) for f in range(F)]
    r = oracle.bwd_update(tabs, "f32", states, dims, t2t, indices, offsets, B, grad, 0.01, 1e-8)
    tab = _table_of_pos(F, B, offsets)
    touched = set(zip(tab.tolist(), indices.tolist()))
    assert set(zip(r["key_table"].tolist(), r["key_row"].tolist())) == touched
    # duplicates are summed first, then ONE step: state rises by mean(G^2) exactly once
    for i, (f, row) in enumerate(zip(r["key_table"], r["key_row"])):
        D = dims[f]
        assert r["D_of"][i] == D
        ms = (r["G"][i, :D] ** 2).mean()
        np.testing.assert_allclose(r["new_state"][i], float(states[f][row]) + ms, rtol=1e-14)
