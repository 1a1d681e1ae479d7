"""Host stages of the Tower Partitioner (paper Sec. 3.3) through the C ABI against the oracle:
distance + Adam embedding, constrained K-means.  They run on the host, so no GPU is needed."""

import numpy as np
import pytest

import paper_2403_00877_amd as dmt
from paper_2403_00877_amd import binding
from oracle import tp


def _sym_interaction(rng, F):
    A = rng.uniform(0, 1, size=(F, F))
    I = (A + A.T) / 2
    np.fill_diagonal(I, 1.0)
    return I.astype(np.float32)


@pytest.mark.parametrize("F,n,strategy,seed", [(8, 2, "coherent", 0), (26, 2, "diverse", 1),
                                               (64, 2, "coherent", 2), (13, 3, "diverse", 3),
                                               (2, 1, "coherent", 4), (1, 2, "diverse", 5)])
def test_embed_matches_the_oracle(F, n, strategy, seed):
    rng = np.random.default_rng(seed)
    I = _sym_interaction(rng, F)
    x0 = rng.normal(size=(F, n))
    for steps in (0, 1, 40):
        x, stress = dmt.dmt_tp_embed(I, strategy, n, steps, 0.05, x0)
        ref, ref_stress = tp.tp_embed(tp.tp_distance(I, strategy), x0, steps, 0.05)
        # float64 on both sides, sums taken in a different order
        np.testing.assert_allclose(x, ref, rtol=1e-9, atol=1e-11)
        assert stress == pytest.approx(ref_stress, rel=1e-9, abs=1e-18)


def test_embed_reads_only_below_the_diagonal_and_lowers_the_stress():
    rng = np.random.default_rng(6)
    F = 20
    I = _sym_interaction(rng, F)
    x0 = rng.normal(size=(F, 2))
    x, stress = dmt.dmt_tp_embed(I, "coherent", 2, 300, 0.02, x0)
    junk = I + np.triu(rng.normal(size=(F, F))).astype(np.float32)
    x2, stress2 = dmt.dmt_tp_embed(junk, "coherent", 2, 300, 0.02, x0)
    np.testing.assert_array_equal(x, x2)
    assert stress == stress2
    assert stress < 0.5 * tp.tp_stress(x0, tp.tp_distance(I, "coherent"))
    assert stress == pytest.approx(tp.tp_stress(x, tp.tp_distance(I, "coherent")), rel=1e-10)


@pytest.mark.parametrize("F,T,ratio,seed", [(64, 8, 1.0, 0), (26, 8, 1.0, 1), (26, 8, 2.0, 2),
                                            (40, 5, 1.5, 3), (12, 12, 1.0, 4), (9, 1, 1.0, 5),
                                            (128, 16, 1.0, 6), (30, 4, 8.0, 7)])
def test_kmeans_matches_the_oracle(F, T, ratio, seed):
    rng = np.random.default_rng(seed)
    x = rng.normal(size=(F, 2))
    x[: F // 3] += 4.0                     # an uneven cloud, so that the size bounds bind
    c0 = x[rng.choice(F, T, replace=False)]
    labels, centres, it = dmt.dmt_tp_kmeans(x, T, ratio, c0)
    ref_labels, ref_centres, ref_it = tp.tp_kmeans(x, c0, ratio)
    np.testing.assert_array_equal(labels, ref_labels)
    np.testing.assert_allclose(centres, ref_centres, rtol=1e-12, atol=1e-13)
    assert it == ref_it
    sizes = np.bincount(labels, minlength=T)
    smin, smax = tp.tp_size_bounds(F, T, ratio)
    assert sizes.min() >= smin and sizes.max() <= smax


def test_kmeans_single_assignment_step_is_the_constrained_optimum():
    rng = np.random.default_rng(8)
    for F, T in ((7, 3), (10, 2), (9, 3)):
        x = rng.normal(size=(F, 2))
        x[:4] += 3.0
        c0 = rng.normal(size=(T, 2))
        labels, centres, it = dmt.dmt_tp_kmeans(x, T, 1.0, c0, max_iter=1)
        assert it == 1
        smin, smax = tp.tp_size_bounds(F, T, 1.0)
        np.testing.assert_array_equal(labels, tp.tp_constrained_assign(x, c0, smin, smax))
        for h in range(T):
            np.testing.assert_allclose(centres[h], x[labels == h].mean(axis=0), atol=1e-13)


def test_partition_on_planted_groups_through_the_host_stages():
    # interaction matrix from the oracle here (the device stage has its own GPU tests)
    rng = np.random.default_rng(9)
    B, G, per, N = 200, 4, 4, 16
    base = rng.normal(size=(B, G, 1, N))
    R = (base + 0.3 * rng.normal(size=(B, G, per, N))).reshape(B, G * per, N)
    group = np.repeat(np.arange(G), per)
    I = tp.tp_interaction(R).astype(np.float32)
    x0 = rng.normal(size=(G * per, 2))
    x, _ = dmt.dmt_tp_embed(I, "coherent", 2, 1500, 0.02, x0)
    labels, _, _ = dmt.dmt_tp_kmeans(x, G, 1.0, x[[0, 4, 8, 12]])
    for h in range(G):
        assert len(set(group[labels == h])) == 1
    x, _ = dmt.dmt_tp_embed(I, "diverse", 2, 1500, 0.02, x0)
    labels, _, _ = dmt.dmt_tp_kmeans(x, per, 1.0, x[[0, 1, 2, 3]])
    for h in range(per):
        assert sorted(group[labels == h]) == list(range(G))


def test_host_stages_reject_bad_arguments():
    lib = binding._lib
    I = np.eye(4, dtype=np.float32)
    x = np.zeros((4, 2))
    out = np.zeros((4, 2))
    lab = np.zeros(4, dtype=np.int32)
    EINVAL = 1

    def embed(I_=I, F=4, strat=0, n=2, steps=1, lr=0.1, x0=x, xo=out):
        return lib.dmt_tp_embed(None if I_ is None else I_.ctypes.data, F, strat, n, steps, lr,
                                None if x0 is None else x0.ctypes.data,
                                None if xo is None else xo.ctypes.data, None)
    assert embed() == 0
    assert embed(I_=None) == EINVAL and embed(x0=None) == EINVAL and embed(xo=None) == EINVAL
    assert embed(F=0) == EINVAL and embed(n=0) == EINVAL and embed(steps=-1) == EINVAL
    assert embed(lr=0.0) == EINVAL and embed(lr=float("nan")) == EINVAL and embed(strat=2) == EINVAL

    def kmeans(x_=x, F=4, n=2, T=2, ratio=1.0, c0=x, iters=5, lab_=lab):
        return lib.dmt_tp_kmeans(None if x_ is None else x_.ctypes.data, F, n, T, ratio,
                                 None if c0 is None else c0.ctypes.data, iters,
                                 None if lab_ is None else lab_.ctypes.data, None, None)
    assert kmeans() == 0
    assert kmeans(x_=None) == EINVAL and kmeans(c0=None) == EINVAL and kmeans(lab_=None) == EINVAL
    assert kmeans(T=0) == EINVAL and kmeans(T=5) == EINVAL and kmeans(ratio=0.5) == EINVAL
    assert kmeans(ratio=float("nan")) == EINVAL and kmeans(iters=0) == EINVAL and kmeans(F=0) == EINVAL
