"""Pins of the Tower Partitioner oracle (oracle/tp.py; paper Sec. 3.3) to things other than itself:
hand cases, brute force on tiny inputs, central differences, torch's autograd and Adam, scipy's
pdist, and planted configurations whose answer is known."""
import itertools
import math

import numpy as np
import pytest
import torch
from scipy.spatial.distance import pdist, squareform

from oracle import tp


# ------------------------------------------------------------------ interaction matrix

def test_interaction_hand_cases():
    # one sample, three features in the plane: e1, 2 e1 (same direction), e2, and -3 e1
    R = np.array([[[1.0, 0.0], [2.0, 0.0], [0.0, 5.0], [-3.0, 0.0]]])
    I = tp.tp_interaction(R)
    expect = np.array([[1, 1, 0, 1], [1, 1, 0, 1], [0, 0, 1, 0], [1, 1, 0, 1]], dtype=float)
    np.testing.assert_allclose(I, expect, atol=1e-15)


def test_interaction_takes_the_absolute_value_of_the_batch_mean():
    # features 0 and 1 agree in half of the batch and oppose in the other half: the mean of the
    # cosines is 0 and so is I (the mean of absolute cosines would be 1); a 3:1 split gives 1/2
    a = np.array([1.0, 2.0, -1.0])
    R = np.stack([np.stack([a, a]), np.stack([a, -a])])
    assert tp.tp_interaction(R)[0, 1] == pytest.approx(0.0, abs=1e-15)
    R = np.stack([np.stack([a, -a])] * 3 + [np.stack([a, a])])
    assert tp.tp_interaction(R)[0, 1] == pytest.approx(0.5, abs=1e-15)


def test_interaction_brute_force_and_invariants():
    rng = np.random.default_rng(1)
    B, F, N = 5, 4, 3
    R = rng.normal(size=(B, F, N))
    R[2, 1] = 0.0                                   # a zero vector: cosine counts as 0
    G = np.zeros((F, F))
    for b in range(B):
        for i in range(F):
            for j in range(F):
                ni = math.sqrt(sum(x * x for x in R[b, i]))
                nj = math.sqrt(sum(x * x for x in R[b, j]))
                if ni > 0 and nj > 0:
                    G[i, j] += sum(R[b, i, k] * R[b, j, k] for k in range(N)) / (ni * nj)
    I = tp.tp_interaction(R)
    np.testing.assert_allclose(I, np.abs(G / B), atol=1e-14)
    np.testing.assert_allclose(I, I.T, atol=0)
    assert I.min() >= 0 and I.max() <= 1 + 1e-15
    assert I[0, 0] == pytest.approx(1.0) and I[1, 1] == pytest.approx((B - 1) / B)
    # cosine does not see the length of a vector
    scale = rng.uniform(0.1, 10, size=(B, F, 1))
    np.testing.assert_allclose(tp.tp_interaction(R * scale), I, atol=1e-14)


def test_interaction_of_noisy_copies_of_group_directions():
    # features of one group share a direction per sample, groups are independent: I is near 1
    # inside a group and near 0 (order 1/sqrt(B N)) across groups
    rng = np.random.default_rng(2)
    B, G, per, N = 400, 3, 4, 32
    base = rng.normal(size=(B, G, 1, N))
    R = (base + 0.05 * rng.normal(size=(B, G, per, N))).reshape(B, G * per, N)
    I = tp.tp_interaction(R)
    same = np.kron(np.eye(G), np.ones((per, per))) > 0
    assert I[same].min() > 0.99
    assert I[~same].max() < 5 / math.sqrt(B * N)


def test_distance_strategies():
    I = np.array([[1.0, 0.25], [0.25, 1.0]])
    np.testing.assert_array_equal(tp.tp_distance(I, "diverse"), I)
    np.testing.assert_array_equal(tp.tp_distance(I, "coherent"), 1 - I)
    with pytest.raises(ValueError):
        tp.tp_distance(I, "other")


# ------------------------------------------------------------------ Euclidean embedding

def test_stress_matches_pdist_and_a_hand_case():
    # three points on a line at 0, 3, 7 with targets 1, 2, 3 for the pairs (1,0), (2,0), (2,1)
    X = np.array([[0.0, 0.0], [3.0, 0.0], [7.0, 0.0]])
    D = np.zeros((3, 3))
    D[1, 0], D[2, 0], D[2, 1] = 1.0, 2.0, 3.0
    assert tp.tp_stress(X, D) == pytest.approx((3 - 1) ** 2 + (7 - 2) ** 2 + (4 - 3) ** 2)
    rng = np.random.default_rng(3)
    X = rng.normal(size=(9, 2))
    Dm = squareform(pdist(rng.normal(size=(9, 4))))
    d = squareform(pdist(X))
    iu = np.triu_indices(9, 1)
    assert tp.tp_stress(X, Dm) == pytest.approx(((d[iu] - Dm[iu]) ** 2).sum(), rel=1e-13)
    # only the entries below the diagonal are read
    junk = Dm + np.triu(rng.normal(size=(9, 9)))
    assert tp.tp_stress(X, junk) == tp.tp_stress(X, Dm)


def test_stress_gradient_against_central_differences_and_autograd():
    rng = np.random.default_rng(4)
    F, n = 7, 2
    X = rng.normal(size=(F, n))
    D = np.abs(rng.normal(size=(F, F)))
    g = tp.tp_stress_grad(X, D)
    h = 1e-6
    for i in range(F):
        for k in range(n):
            Xp, Xm = X.copy(), X.copy()
            Xp[i, k] += h
            Xm[i, k] -= h
            fd = (tp.tp_stress(Xp, D) - tp.tp_stress(Xm, D)) / (2 * h)
            assert g[i, k] == pytest.approx(fd, rel=1e-6, abs=1e-7)
    Xt = torch.tensor(X, requires_grad=True)
    loss = _torch_stress(Xt, torch.tensor(D))
    loss.backward()
    np.testing.assert_allclose(g, Xt.grad.numpy(), rtol=1e-12, atol=1e-13)


def _torch_stress(Xt, Dt):
    F = Xt.shape[0]
    i, j = torch.tril_indices(F, F, -1)
    d = (Xt[i] - Xt[j]).pow(2).sum(dim=1).sqrt()
    return (d - Dt[i, j]).pow(2).sum()


def test_stress_gradient_vanishes_at_an_exact_embedding_and_for_coincident_points():
    rng = np.random.default_rng(5)
    P = rng.normal(size=(6, 2))
    D = squareform(pdist(P))
    np.testing.assert_allclose(tp.tp_stress_grad(P, D), 0, atol=1e-14)
    assert tp.tp_stress(P, D) == pytest.approx(0, abs=1e-28)
    # two coincident points pull on nothing between themselves
    X = np.array([[1.0, 1.0], [1.0, 1.0]])
    D2 = np.array([[0.0, 0.0], [0.5, 0.0]])
    np.testing.assert_array_equal(tp.tp_stress_grad(X, D2), 0)
    assert tp.tp_stress(X, D2) == pytest.approx(0.25)


def test_embed_follows_torch_adam_step_for_step():
    rng = np.random.default_rng(6)
    F, n, steps, lr = 8, 2, 25, 0.05
    X0 = rng.normal(size=(F, n))
    D = np.abs(rng.normal(size=(F, F)))
    X, stress = tp.tp_embed(D, X0, steps, lr)
    Xt = torch.tensor(X0, requires_grad=True)
    opt = torch.optim.Adam([Xt], lr=lr, betas=(0.9, 0.999), eps=1e-8)
    Dt = torch.tensor(D)
    for _ in range(steps):
        opt.zero_grad()
        _torch_stress(Xt, Dt).backward()
        opt.step()
    np.testing.assert_allclose(X, Xt.detach().numpy(), rtol=1e-9, atol=1e-11)
    assert stress == pytest.approx(float(_torch_stress(Xt, Dt).detach()), rel=1e-9)
    # zero steps leave the start where it is
    X_same, s0 = tp.tp_embed(D, X0, 0, lr)
    np.testing.assert_array_equal(X_same, X0)
    assert s0 == pytest.approx(tp.tp_stress(X0, D))


def test_embed_recovers_a_planar_configuration():
    # distances that a 2-D configuration realises exactly: Adam brings the stress to ~0 and
    # the pairwise distances of the result are the targets (the coordinates themselves are
    # only fixed up to a rigid motion)
    rng = np.random.default_rng(7)
    P = rng.uniform(-1, 1, size=(10, 2))
    D = squareform(pdist(P))
    X0 = P + 0.2 * rng.normal(size=P.shape)
    s0 = tp.tp_stress(X0, D)
    X, stress = tp.tp_embed(D, X0, 3000, 0.01)
    assert stress < 1e-6 * s0
    np.testing.assert_allclose(squareform(pdist(X)), D, atol=1e-3)


# ------------------------------------------------------------------ constrained K-means

def test_size_bounds():
    assert tp.tp_size_bounds(64, 8, 1) == (8, 8)
    assert tp.tp_size_bounds(256, 16, 1) == (16, 16)
    assert tp.tp_size_bounds(26, 8, 1) == (3, 4)          # the paper's 26 features on 8 towers
    assert tp.tp_size_bounds(26, 8, 2) == (3, 6)
    assert tp.tp_size_bounds(26, 26, 1) == (1, 1)
    assert tp.tp_size_bounds(26, 1, 1) == (26, 26)
    assert tp.tp_size_bounds(10, 3, 1.5) == (3, 4)
    for F, T, R in itertools.product(range(1, 40), range(1, 12), (1, 1.25, 1.5, 2, 3, 8)):
        if T > F:
            continue
        smin, smax = tp.tp_size_bounds(F, T, R)
        assert 1 <= smin <= F // T and smax >= -(-F // T)          # T groups fit inside the bounds
        # the ratio holds whenever integers allow it at all
        assert smax <= R * smin + 1e-9 or (smin == F // T and smax == -(-F // T))
    with pytest.raises(ValueError):
        tp.tp_size_bounds(3, 4, 1)
    with pytest.raises(ValueError):
        tp.tp_size_bounds(8, 2, 0.5)


def _brute_assign(X, C, smin, smax):
    F, T = len(X), len(C)
    best, best_cost = None, None
    for lab in itertools.product(range(T), repeat=F):
        counts = [lab.count(h) for h in range(T)]
        if min(counts) < smin or max(counts) > smax:
            continue
        cost = sum(((X[i] - C[lab[i]]) ** 2).sum() for i in range(F))
        if best_cost is None or cost < best_cost:
            best, best_cost = lab, cost
    return np.array(best), best_cost


@pytest.mark.parametrize("F,T,smin,smax,seed", [(6, 3, 2, 2, 0), (7, 2, 3, 4, 1), (7, 3, 2, 3, 2),
                                                 (8, 2, 1, 7, 3), (6, 3, 1, 4, 4), (5, 5, 1, 1, 5)])
def test_constrained_assignment_against_brute_force(F, T, smin, smax, seed):
    rng = np.random.default_rng(seed)
    X = rng.normal(size=(F, 2))
    X[: F // 2] += 3.0          # an uneven cloud, so that the size bounds bind
    C = rng.normal(size=(T, 2))
    lab = tp.tp_constrained_assign(X, C, smin, smax)
    ref, ref_cost = _brute_assign(X, C, smin, smax)
    np.testing.assert_array_equal(lab, ref)
    assert tp.tp_kmeans_cost(X, C, lab) == pytest.approx(ref_cost, rel=1e-12)
    with pytest.raises(ValueError):
        tp.tp_constrained_assign(X, C, F, F)


def test_loose_bounds_give_the_nearest_centre():
    rng = np.random.default_rng(8)
    X = rng.normal(size=(30, 2))
    C = rng.normal(size=(4, 2))
    lab = tp.tp_constrained_assign(X, C, 0, 30)
    d2 = ((X[:, None] - C[None]) ** 2).sum(axis=2)
    np.testing.assert_array_equal(lab, d2.argmin(axis=1))


def test_kmeans_recovers_planted_balanced_clusters_and_respects_the_ratio():
    rng = np.random.default_rng(9)
    T, per = 4, 6
    centres = np.array([[0, 0], [10, 0], [0, 10], [10, 10]], dtype=float)
    X = (centres[:, None, :] + 0.5 * rng.normal(size=(T, per, 2))).reshape(-1, 2)
    perm = rng.permutation(T * per)
    X = X[perm]
    truth = np.repeat(np.arange(T), per)[perm]
    start = X[[int(np.nonzero(truth == h)[0][0]) for h in range(T)]]
    lab, C, it = tp.tp_kmeans(X, start, 1.0)
    np.testing.assert_array_equal(lab, truth)
    for h in range(T):
        np.testing.assert_allclose(C[h], X[truth == h].mean(axis=0), atol=1e-12)
    # unbalanced cloud (12 + 4 + 4 + 4 points), R = 1: the groups are still 6 each; R = 3 lets
    # the natural grouping through
    Xu = np.concatenate([centres[0] + 0.5 * rng.normal(size=(12, 2))] +
                        [centres[h] + 0.5 * rng.normal(size=(4, 2)) for h in (1, 2, 3)])
    for R in (1.0, 1.5, 3.0):
        lab, C, it = tp.tp_kmeans(Xu, centres, R)
        sizes = np.bincount(lab, minlength=T)
        assert sizes.max() <= R * sizes.min() + 1e-9
    assert sorted(np.bincount(tp.tp_kmeans(Xu, centres, 1.0)[0])) == [6, 6, 6, 6]
    assert sorted(np.bincount(tp.tp_kmeans(Xu, centres, 3.0)[0])) == [4, 4, 4, 12]


def test_kmeans_cost_never_rises():
    rng = np.random.default_rng(10)
    X = rng.normal(size=(26, 2))
    C = X[rng.choice(26, 8, replace=False)]
    smin, smax = tp.tp_size_bounds(26, 8, 1)
    prev = None
    for _ in range(20):
        lab = tp.tp_constrained_assign(X, C, smin, smax)
        c_assign = tp.tp_kmeans_cost(X, C, lab)
        assert prev is None or c_assign <= prev + 1e-12
        C = np.stack([X[lab == h].mean(axis=0) for h in range(8)])
        prev = tp.tp_kmeans_cost(X, C, lab)
        assert prev <= c_assign + 1e-12
    lab2, C2, it = tp.tp_kmeans(X, X[:8], 1.0)
    assert sorted(np.bincount(lab2)) == [3, 3, 3, 3, 3, 3, 4, 4]
    assert it < 100


def test_partition_end_to_end_on_planted_groups():
    # coherent strategy: features that move together land in one tower; diverse strategy: every
    # tower gets one feature of each planted group
    rng = np.random.default_rng(11)
    B, G, per, N = 256, 4, 4, 16
    base = rng.normal(size=(B, G, 1, N))
    R = (base + 0.3 * rng.normal(size=(B, G, per, N))).reshape(B, G * per, N)
    group = np.repeat(np.arange(G), per)
    F = G * per
    X0 = rng.normal(size=(F, 2))
    res = tp.tp_partition(R, G, "coherent", X0, [0, 4, 8, 12], 1500, 0.02)
    for h in range(G):
        assert len(set(group[res["labels"] == h])) == 1
    assert sorted(np.bincount(res["labels"])) == [per] * G
    res = tp.tp_partition(R, per, "diverse", X0, [0, 1, 2, 3], 1500, 0.02)
    for h in range(per):
        assert sorted(group[res["labels"] == h]) == list(range(G))
