"""Tower Partitioner, CPU oracle.  TEST INFRASTRUCTURE ONLY.

Only tests and the benchmark's CPU-baseline leg may import this module; the
product package never does, and nothing here touches the HIP library.

The Tower Partitioner (paper Sec. 3.3) turns the embeddings a model produces
for a batch into a balanced feature -> tower map in four steps, each written
out here as the paper defines it, in float64:

  1. interaction matrix: the cosine kernel between the normalised embeddings
     of features i and j, averaged over the batch (the mean of R R^T along the
     batch dimension, R of shape (B, F, N)), then the absolute value;
  2. distance matrix D = f(I): f(I) = I (diverse strategy) or 1 - I (coherent);
  3. coordinates X_i in R^n (n < N) that minimise the sum over pairs j < i of
     (||X_i - X_j||_2 - D(i, j))^2, by Adam from given start coordinates;
  4. constrained K-means (Bradley, Bennett and Demiriz 2000: Lloyd's iteration
     whose assignment step is the minimum-cost assignment under bounds on the
     cluster sizes), with the bound that the largest group holds at most R
     times as many features as the smallest.

Library steps: numpy's matmul / einsum, scipy's linear_sum_assignment for the
assignment step.  The random numbers the method draws (start coordinates, start
centres) are arguments.  Pinned in tests/test_oracle_tp.py against hand cases,
brute force on tiny inputs, central differences, torch's autograd and Adam, and
planted configurations.
"""
from __future__ import annotations

import math
from typing import Tuple

import numpy as np
from scipy.optimize import linear_sum_assignment


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


# ---------------------------------------------------------------- step 1: interaction

def tp_interaction(R) -> np.ndarray:
    """I = | mean over b of  Rn_b Rn_b^T |,  Rn_b[f] = R_b[f] / ||R_b[f]||_2  (Sec. 3.3).

    `R` is (B, F, N).  A zero vector has no direction: it is left zero, so its
    cosine with anything counts as 0 in the batch mean.
    """
    R = _f64(R)
    B = R.shape[0]
    norm = np.sqrt((R * R).sum(axis=2, keepdims=True))
    Rn = np.divide(R, norm, out=np.zeros_like(R), where=norm > 0)
    G = np.einsum("bik,bjk->ij", Rn, Rn) / B
    return np.abs(G)


# ---------------------------------------------------------------- step 2: distance

def tp_distance(I, strategy: str) -> np.ndarray:
    """D = f(I): "diverse" f(I) = I, "coherent" f(I) = 1 - I  (Sec. 3.3)."""
    I = _f64(I)
    if strategy == "diverse":
        return I.copy()
    if strategy == "coherent":
        return 1.0 - I
    raise ValueError(strategy)


# ---------------------------------------------------------------- step 3: embedding

def _pair_targets(D) -> np.ndarray:
    """D(i, j) for j < i, mirrored so that entry [i][j] and [j][i] both hold the pair's target."""
    L = np.tril(_f64(D), -1)
    return L + L.T


def tp_stress(X, D) -> float:
    """sum over i, over j < i, of (||X_i - X_j||_2 - D(i, j))^2  (Sec. 3.3)."""
    X = _f64(X)
    diff = X[:, None, :] - X[None, :, :]
    d = np.sqrt((diff * diff).sum(axis=2))
    e = np.tril(d - _pair_targets(D), -1)
    return float((e * e).sum())


def tp_stress_grad(X, D) -> np.ndarray:
    """Gradient of tp_stress in X:  row i = sum over j != i of
    2 (d_ij - D(i, j)) (X_i - X_j) / d_ij ;  a pair of coincident points (d_ij = 0)
    contributes nothing."""
    X = _f64(X)
    diff = X[:, None, :] - X[None, :, :]
    d = np.sqrt((diff * diff).sum(axis=2))
    c = np.divide(2.0 * (d - _pair_targets(D)), d, out=np.zeros_like(d), where=d > 0)
    return (c[:, :, None] * diff).sum(axis=1)


def tp_embed(D, X0, steps: int, lr: float, beta1: float = 0.9, beta2: float = 0.999,
             eps: float = 1e-8) -> Tuple[np.ndarray, float]:
    """`steps` iterations of Adam (Kingma and Ba, with bias correction) on tp_stress from X0.
    Returns the coordinates and their stress."""
    X = _f64(X0).copy()
    m = np.zeros_like(X)
    v = np.zeros_like(X)
    for t in range(1, steps + 1):
        g = tp_stress_grad(X, D)
        m = beta1 * m + (1.0 - beta1) * g
        v = beta2 * v + (1.0 - beta2) * g * g
        mhat = m / (1.0 - beta1 ** t)
        vhat = v / (1.0 - beta2 ** t)
        X = X - lr * mhat / (np.sqrt(vhat) + eps)
    return X, tp_stress(X, D)


# ---------------------------------------------------------------- step 4: constrained K-means

def tp_size_bounds(F: int, T: int, R: float) -> Tuple[int, int]:
    """Bounds (smin, smax) on the group sizes so that max <= R * min holds for the result.

    With a floor of s on every group the largest group can hold F - (T - 1) s, which is at
    most R s once s >= F / (T - 1 + R); smin is that floor, capped at floor(F / T) so that T
    groups fit.  smax = floor(R * smin), but never below ceil(F / T) or nothing would fit: with
    R = 1 and T not dividing F the groups are as even as integers allow (floor and ceil of F / T).
    """
    if not (1 <= T <= F) or R < 1:
        raise ValueError("need 1 <= T <= F and R >= 1")
    smin = min(math.ceil(F / (T - 1 + R) - 1e-12), F // T)
    smax = max(math.floor(R * smin + 1e-12), -(-F // T))
    return smin, smax


def tp_constrained_assign(X, C, smin: int, smax: int) -> np.ndarray:
    """The assignment step: labels minimising sum_i ||X_i - C_label(i)||^2 subject to
    smin <= |group| <= smax for every group.

    Written as a square assignment problem: group h offers smax slots, of which the first smin
    must be taken; T smax - F dummy points cost nothing in an optional slot and more than any
    complete assignment of real points in a mandatory one.
    """
    X, C = _f64(X), _f64(C)
    F, T = X.shape[0], C.shape[0]
    if T * smin > F or T * smax < F:
        raise ValueError("size bounds leave no feasible assignment")
    d2 = ((X[:, None, :] - C[None, :, :]) ** 2).sum(axis=2)        # [F][T]
    n = T * smax
    big = 1.0 + d2.sum()
    cost = np.zeros((n, n))
    slot_group = np.repeat(np.arange(T), smax)
    slot_mandatory = np.tile(np.arange(smax) < smin, T)
    cost[:F, :] = d2[:, slot_group]
    cost[F:, :] = np.where(slot_mandatory, big, 0.0)[None, :]
    rows, cols = linear_sum_assignment(cost)
    labels = np.empty(F, dtype=np.int32)
    for r, c in zip(rows, cols):
        if r < F:
            labels[r] = slot_group[c]
    return labels


def tp_kmeans_cost(X, C, labels) -> float:
    X, C = _f64(X), _f64(C)
    return float(((X - C[np.asarray(labels)]) ** 2).sum())


def tp_kmeans(X, C0, R: float, max_iter: int = 100) -> Tuple[np.ndarray, np.ndarray, int]:
    """Constrained K-means from the centres C0 (T of them): assign under the size bounds of
    tp_size_bounds, move every centre to the mean of its group, until the labels stop changing
    (or max_iter assignment steps).  Returns (labels, centres, assignment steps taken)."""
    X = _f64(X)
    C = _f64(C0).copy()
    F, T = X.shape[0], C.shape[0]
    smin, smax = tp_size_bounds(F, T, R)
    labels = None
    it = 0
    while it < max_iter:
        new = tp_constrained_assign(X, C, smin, smax)
        it += 1
        if labels is not None and np.array_equal(new, labels):
            break
        labels = new
        for h in range(T):
            members = X[labels == h]
            if len(members):
                C[h] = members.mean(axis=0)
    return labels, C, it


def tp_partition(R, T: int, strategy: str, X0, C0_index, steps: int, lr: float,
                 ratio: float = 1.0, max_iter: int = 100):
    """All four steps: embeddings (B, F, N) -> feature -> tower labels.  The start centres are
    the embedded coordinates of the features listed in C0_index."""
    I = tp_interaction(R)
    D = tp_distance(I, strategy)
    X, stress = tp_embed(D, X0, steps, lr)
    labels, C, it = tp_kmeans(X, X[np.asarray(C0_index)], ratio, max_iter)
    return dict(I=I, D=D, X=X, stress=stress, labels=labels, centres=C, iterations=it)
