"""Pins of the Tower Module backward oracle (oracle/tm_bwd.py).

The backward is pinned against something other than itself: central differences of the FORWARD
oracle (oracle.tm_linear / tm_dot_linear / tm_cross_linear, pinned in test_oracle_tm.py),
closed forms, and hand-computed cases.  A dropped term, a wrong sign, a transposed operand or
a swapped pair index fails at least one of them.
"""
import numpy as np
import pytest

import oracle
from oracle import tm_bwd


def _numeric_grad(f, a, h=1e-6):
    """Central differences of the scalar function f with respect to every entry of a."""
    g = np.zeros_like(a)
    flat, gf = a.reshape(-1), g.reshape(-1)
    for i in range(flat.size):
        keep = flat[i]
        flat[i] = keep + h
        up = f()
        flat[i] = keep - h
        dn = f()
        flat[i] = keep
        gf[i] = (up - dn) / (2 * h)
    return g


def _close(a, b, tol=2e-7):
    scale = max(1.0, float(np.max(np.abs(b))))
    assert np.max(np.abs(a - b)) <= tol * scale, (np.max(np.abs(a - b)), scale)


@pytest.mark.parametrize("relu", [False, True])
def test_linear_against_central_differences(relu):
    rng = np.random.default_rng(1)
    B, K, O = 5, 7, 4
    x, W, b = rng.normal(size=(B, K)), rng.normal(size=(O, K)), rng.normal(size=O)
    R = rng.normal(size=(B, O))                      # L = sum(y * R), so dL/dy = R
    loss = lambda: float(np.sum(oracle.tm_linear(x, W, b, relu) * R))
    dx, dW, db = tm_bwd.tm_linear_bwd(x, W, b, R, relu)
    _close(dx, _numeric_grad(loss, x))
    _close(dW, _numeric_grad(loss, W))
    _close(db, _numeric_grad(loss, b))


def test_linear_closed_forms():
    rng = np.random.default_rng(2)
    x, dy = rng.normal(size=(6, 5)), rng.normal(size=(6, 5))
    dx, dW, db = tm_bwd.tm_linear_bwd(x, np.eye(5), np.zeros(5), dy)
    assert np.array_equal(dx, dy)                    # identity weights pass the gradient through
    _close(dW, dy.T @ x)
    _close(db, dy.sum(0))
    # ReLU with a bias far below zero switches every output off
    dx, dW, db = tm_bwd.tm_linear_bwd(x, np.eye(5), np.full(5, -100.0), dy, relu=True)
    assert not dx.any() and not dW.any() and not db.any()


def test_linear_hand_computed():
    # y = [2 x0 + 3 x1 + 1], one sample x = (4, 5), dy = 10
    dx, dW, db = tm_bwd.tm_linear_bwd([[4.0, 5.0]], [[2.0, 3.0]], [1.0], [[10.0]])
    assert dx.tolist() == [[20.0, 30.0]] and dW.tolist() == [[40.0, 50.0]] and db.tolist() == [10.0]


@pytest.mark.parametrize("nf,n", [(2, 1), (3, 2), (4, 3)])
def test_dot_linear_against_central_differences(nf, n):
    rng = np.random.default_rng(3)
    B, O = 4, 3
    kin = nf * (nf - 1) // 2 + nf * n
    x, W, b = rng.normal(size=(B, nf * n)), rng.normal(size=(O, kin)), rng.normal(size=O)
    R = rng.normal(size=(B, O))
    loss = lambda: float(np.sum(oracle.tm_dot_linear(x, nf, W, b) * R))
    dx, dW, db = tm_bwd.tm_dot_linear_bwd(x, nf, W, b, R)
    _close(dx, _numeric_grad(loss, x))
    _close(dW, _numeric_grad(loss, W))
    _close(db, _numeric_grad(loss, b))


def test_dot_linear_hand_computed_two_scalar_features():
    # nf = 2, n = 1: z = (x0 x1, x0, x1), y = 2 x0 x1 + 3 x0 + 5 x1 + 7; at x = (4, 6), dy = 1:
    # dy/dx0 = 2 x1 + 3 = 15, dy/dx1 = 2 x0 + 5 = 13, dW = z = (24, 4, 6), db = 1
    dx, dW, db = tm_bwd.tm_dot_linear_bwd([[4.0, 6.0]], 2, [[2.0, 3.0, 5.0]], [7.0], [[1.0]])
    assert dx.tolist() == [[15.0, 13.0]] and dW.tolist() == [[24.0, 4.0, 6.0]] and db.tolist() == [1.0]


def test_dot_pair_order_is_row_major():
    # three scalar features; only the weight of pair (0, 2), the second dot column, is non-zero:
    # y = x0 x2, so the gradient is (x2, 0, x0)
    W = np.zeros((1, 3 + 3))
    W[0, 1] = 1.0
    dx, _, _ = tm_bwd.tm_dot_linear_bwd([[2.0, 3.0, 5.0]], 3, W, [0.0], [[1.0]])
    assert dx.tolist() == [[5.0, 0.0, 2.0]]


@pytest.mark.parametrize("layers", [1, 2, 3])
def test_cross_linear_against_central_differences(layers):
    rng = np.random.default_rng(4)
    B, d, O = 3, 5, 2
    x = rng.normal(size=(B, d))
    Wc = [0.3 * rng.normal(size=(d, d)) for _ in range(layers)]
    bc = [rng.normal(size=d) for _ in range(layers)]
    W, b = rng.normal(size=(O, d)), rng.normal(size=O)
    R = rng.normal(size=(B, O))
    loss = lambda: float(np.sum(oracle.tm_cross_linear(x, Wc, bc, W, b) * R))
    dx, dWc, dbc, dW, db = tm_bwd.tm_cross_linear_bwd(x, Wc, bc, W, b, R)
    _close(dx, _numeric_grad(loss, x), 1e-6)
    for l in range(layers):
        _close(dWc[l], _numeric_grad(loss, Wc[l]), 1e-6)
        _close(dbc[l], _numeric_grad(loss, bc[l]), 1e-6)
    _close(dW, _numeric_grad(loss, W), 1e-6)
    _close(db, _numeric_grad(loss, b), 1e-6)


def test_cross_scalar_by_hand():
    # d = 1, one layer: x1 = x (w x + c) + x, y = v x1 + e.  At x = 2, w = 3, c = 1, v = 5:
    # x1 = 2 * 7 + 2 = 16; dy = 1: dx1 = 5, du = dx1 * x = 10, dw = du * x = 20, dc = 10,
    # dx = du * w + dx1 (x_l path) + dx1 * u (x0 factor) = 30 + 5 + 35 = 70 = d/dx [5 (3x^2 + 2x)]
    dx, dWc, dbc, dW, db = tm_bwd.tm_cross_linear_bwd([[2.0]], [[[3.0]]], [[1.0]], [[5.0]], [0.0], [[1.0]])
    assert dx.tolist() == [[70.0]]
    assert dWc[0].tolist() == [[20.0]] and dbc[0].tolist() == [10.0]
    assert dW.tolist() == [[16.0]] and db.tolist() == [1.0]


def test_cross_zero_weights_reduce_to_a_linear_layer():
    # W_l = 0, b_l = 0: every cross layer is the identity, so the module is its projection
    rng = np.random.default_rng(5)
    x, W, b, dy = rng.normal(size=(4, 3)), rng.normal(size=(2, 3)), rng.normal(size=2), rng.normal(size=(4, 2))
    Z, z = [np.zeros((3, 3))] * 2, [np.zeros(3)] * 2
    dx, dWc, dbc, dW, db = tm_bwd.tm_cross_linear_bwd(x, Z, z, W, b, dy)
    lx, lW, lb = tm_bwd.tm_linear_bwd(x, W, b, dy)
    _close(dx, lx)
    _close(dW, lW)
    _close(db, lb)


def test_dlrm_module_against_central_differences():
    rng = np.random.default_rng(6)
    B, F, N, pD, cD = 4, 3, 2, 3, 2
    x = rng.normal(size=(B, F * N))
    Wp, bp = rng.normal(size=(pD, F * N)), rng.normal(size=pD)
    Wf, bf = rng.normal(size=(cD, N)), rng.normal(size=cD)
    R = rng.normal(size=(B, pD + F * cD))
    loss = lambda: float(np.sum(oracle.tm_dlrm(x, F, Wp, bp, Wf, bf) * R))
    dx, dWp, dbp, dWf, dbf = tm_bwd.tm_dlrm_bwd(x, F, Wp, bp, Wf, bf, R)
    _close(dx, _numeric_grad(loss, x))
    _close(dWp, _numeric_grad(loss, Wp))
    _close(dbp, _numeric_grad(loss, bp))
    _close(dWf, _numeric_grad(loss, Wf))
    _close(dbf, _numeric_grad(loss, bf))


def test_dlrm_module_hand_computed_shared_weights():
    # |F| = 2, N = 1, no flat outputs worth mentioning (pD = 1 with zero weight), cD = 1:
    # y = (b, w x0 + c, w x1 + c); dy = (0, 2, 3): dw = 2 x0 + 3 x1, dc = 5, dx = (2 w, 3 w)
    dx, dWp, dbp, dWf, dbf = tm_bwd.tm_dlrm_bwd([[4.0, 5.0]], 2, [[0.0, 0.0]], [1.0], [[7.0]], [0.5],
                                                [[0.0, 2.0, 3.0]])
    assert dx.tolist() == [[14.0, 21.0]]
    assert dWf.tolist() == [[23.0]] and dbf.tolist() == [5.0]
    assert dWp.tolist() == [[0.0, 0.0]] and dbp.tolist() == [0.0]


@pytest.mark.parametrize("layers", [1, 2])
def test_lowrank_cross_against_central_differences(layers):
    rng = np.random.default_rng(7)
    B, d, r, O = 3, 5, 2, 2
    x = rng.normal(size=(B, d))
    Vc = [0.4 * rng.normal(size=(r, d)) for _ in range(layers)]
    Uc = [0.4 * rng.normal(size=(d, r)) for _ in range(layers)]
    bc = [rng.normal(size=d) for _ in range(layers)]
    W, b = rng.normal(size=(O, d)), rng.normal(size=O)
    R = rng.normal(size=(B, O))
    loss = lambda: float(np.sum(oracle.tm_cross_lowrank_linear(x, Vc, Uc, bc, W, b) * R))
    dx, dVc, dUc, dbc, dW, db = tm_bwd.tm_cross_lowrank_linear_bwd(x, Vc, Uc, bc, W, b, R)
    _close(dx, _numeric_grad(loss, x), 1e-6)
    for l in range(layers):
        _close(dVc[l], _numeric_grad(loss, Vc[l]), 1e-6)
        _close(dUc[l], _numeric_grad(loss, Uc[l]), 1e-6)
        _close(dbc[l], _numeric_grad(loss, bc[l]), 1e-6)
    _close(dW, _numeric_grad(loss, W), 1e-6)
    _close(db, _numeric_grad(loss, b), 1e-6)


def test_lowrank_cross_against_the_full_rank_backward():
    # with W_l = U_l V_l the input, bias and projection gradients are those of the full-rank
    # module, and dW_l of the full-rank module factors as dU_l = dW_l V_l^T, dV_l = U_l^T dW_l
    rng = np.random.default_rng(8)
    B, d, r, O = 4, 4, 2, 3
    x = rng.normal(size=(B, d))
    Vc = [0.4 * rng.normal(size=(r, d)) for _ in range(2)]
    Uc = [0.4 * rng.normal(size=(d, r)) for _ in range(2)]
    bc = [rng.normal(size=d) for _ in range(2)]
    W, b, dy = rng.normal(size=(O, d)), rng.normal(size=O), rng.normal(size=(B, O))
    dx, dVc, dUc, dbc, dW, db = tm_bwd.tm_cross_lowrank_linear_bwd(x, Vc, Uc, bc, W, b, dy)
    fx, fWc, fbc, fW, fb = tm_bwd.tm_cross_linear_bwd(x, [U @ V for U, V in zip(Uc, Vc)], bc, W, b, dy)
    _close(dx, fx)
    _close(dW, fW)
    _close(db, fb)
    for l in range(2):
        _close(dbc[l], fbc[l])
        _close(dUc[l], fWc[l] @ Vc[l].T)
        _close(dVc[l], Uc[l].T @ fWc[l])
