"""Pins for the oracle's tower modules (CPU only): library matmul on random
inputs, closed forms and special cases; shapes from the paper's Sec. 4."""
import os

import numpy as np

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def test_linear_against_numpy_matmul():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((37, 20))
    W = rng.standard_normal((11, 20))
    b = rng.standard_normal(11)
    np.testing.assert_allclose(oracle.tm_linear(x, W, b), x @ W.T + b, rtol=1e-12, atol=1e-12)


def test_linear_identity_and_relu():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((9, 6))
    assert np.array_equal(oracle.tm_linear(x, np.eye(6), np.zeros(6)), x)
    y = oracle.tm_linear(x, np.eye(6), np.zeros(6), relu=True)
    assert np.array_equal(y, np.where(x > 0, x, 0.0))
    assert (oracle.tm_linear(-np.abs(x), np.eye(6), np.zeros(6), relu=True) == 0).all()
    # a transposed weight must fail: non-square W picks rows, not columns
    W = np.zeros((2, 6)); W[0, 1] = 1; W[1, 4] = 1
    assert np.array_equal(oracle.tm_linear(x, W, np.array([10.0, 20.0])),
                          np.stack([x[:, 1] + 10, x[:, 4] + 20], axis=1))


def test_dot_terms_count_order_and_values():
    nf, n, B = 8, 16, 5
    rng = np.random.default_rng(2)
    x = rng.standard_normal((B, nf * n))
    kin = nf * (nf - 1) // 2 + nf * n
    assert nf * (nf - 1) // 2 == 28
    W = np.eye(kin)
    y, z = oracle.tm_dot_linear(x, nf, W, np.zeros(kin), return_z=True)
    assert np.array_equal(y, z)                          # identity projection returns z
    assert np.array_equal(z[:, 28:], x)                  # flattened features come after the dots
    gram = np.einsum("bik,bjk->bij", x.reshape(B, nf, n), x.reshape(B, nf, n))
    iu = np.triu_indices(nf, k=1)                        # row-major (i, j), i < j
    np.testing.assert_allclose(z[:, :28], gram[:, iu[0], iu[1]], rtol=1e-12, atol=1e-12)


def test_dot_orthonormal_and_equal_rows():
    nf, n = 4, 4
    x = np.eye(4).reshape(1, 16)                         # orthonormal features
    _, z = oracle.tm_dot_linear(x, nf, np.zeros((1, 22)), np.zeros(1), return_z=True)
    assert (z[0, :6] == 0).all()
    v = np.array([1.0, -2.0, 3.0, 0.5])
    x = np.tile(v, nf).reshape(1, 16)                    # all features equal
    _, z = oracle.tm_dot_linear(x, nf, np.zeros((1, 22)), np.zeros(1), return_z=True)
    assert np.array_equal(z[0, :6], np.full(6, (v * v).sum()))
    # distinguishable pairs: feature i = (i+1) * e_0  ->  dot(i, j) = (i+1)(j+1)
    x = np.zeros((1, nf, n)); x[0, :, 0] = [1, 2, 3, 4]
    _, z = oracle.tm_dot_linear(x.reshape(1, -1), nf, np.zeros((1, 22)), np.zeros(1), return_z=True)
    assert z[0, :6].tolist() == [2, 3, 4, 6, 8, 12]


def test_cross_layer_closed_forms():
    rng = np.random.default_rng(3)
    B, d = 6, 10
    x0 = rng.standard_normal((B, d))
    x = rng.standard_normal((B, d))
    # W = 0, b = 0: the layer is the identity on x
    assert np.array_equal(oracle.cross_layer(x0, x, np.zeros((d, d)), np.zeros(d)), x)
    # W = I, b = 0: x1 = x0*x0 + x0, x2 = x0*x1 + x1
    I = np.eye(d)
    x1 = oracle.cross_layer(x0, x0, I, np.zeros(d))
    np.testing.assert_allclose(x1, x0 * x0 + x0, rtol=1e-15)
    x2 = oracle.cross_layer(x0, x1, I, np.zeros(d))
    np.testing.assert_allclose(x2, x0 * x1 + x1, rtol=1e-15)
    # bias only: xn = x0 * b + x
    b = rng.standard_normal(d)
    np.testing.assert_allclose(oracle.cross_layer(x0, x, np.zeros((d, d)), b), x0 * b + x, rtol=1e-15)
    # general case against numpy
    W = rng.standard_normal((d, d))
    np.testing.assert_allclose(oracle.cross_layer(x0, x, W, b), x0 * (x @ W.T + b) + x, rtol=1e-12)


def test_cross_scalar_recurrence_by_hand():
    # d = 1: x0 = 2, W = [3, -1], b = [0.5, 1]:
    # x1 = 2*(3*2 + 0.5) + 2 = 15 ; x2 = 2*(-1*15 + 1) + 15 = -13 ; y = 4*(-13) + 1 = -51
    y = oracle.tm_cross_linear(np.array([[2.0]]), [np.array([[3.0]]), np.array([[-1.0]])],
                               [np.array([0.5]), np.array([1.0])], np.array([[4.0]]), np.array([1.0]))
    assert y.tolist() == [[-51.0]]


def test_output_shapes_follow_the_listings():
    """Sec. 4: DLRM tower module with c = 0 gives O = p*D; DCN tower module gives
    O = |F|*D.  Table 5 pairs D = 64, 32, 16, 8 (N = 128, c = 1, p = 0) with
    compression ratios 2, 4, 8, 16, so the ratio is input width over output
    width (the printed formula has the fraction upside down)."""
    rows = [[int(v) for v in l.split()] for l in open(os.path.join(GOLD, "table5_compression.txt"))
            if l.strip() and not l.startswith("#")]
    N, F = 128, 26
    for D, cr in rows:
        out_total = F * D * 1                   # c = 1, p = 0: O = D * (c|F| + p) summed over towers
        assert (F * N) / out_total == cr
    B, nf, n, D = 3, 4, 8, 2
    x = np.zeros((B, nf * n))
    assert oracle.tm_linear(x, np.zeros((1 * 16, nf * n)), np.zeros(16)).shape == (B, 16)      # p*D
    y = oracle.tm_cross_linear(x, [np.zeros((nf * n, nf * n))], [np.zeros(nf * n)],
                               np.zeros((nf * D, nf * n)), np.zeros(nf * D))
    assert y.shape == (B, nf * D)


def test_dlrm_module_by_hand_and_against_einsum():
    # Listing 1 with |F| = 2, N = 2, pD = 1, cD = 2 on x = (1, 2 | 3, 4):
    # o1 = 1 + 2 + 3 + 4 + 0.5; feature 0: (1 - 2, 2*1 + 1); feature 1: (3 - 4, 2*3 + 1)
    y = oracle.tm_dlrm([[1.0, 2.0, 3.0, 4.0]], 2, [[1.0, 1.0, 1.0, 1.0]], [0.5],
                       [[1.0, -1.0], [2.0, 0.0]], [0.0, 1.0])
    assert y.tolist() == [[10.5, -1.0, 3.0, -1.0, 7.0]]
    rng = np.random.default_rng(11)
    B, F, N, pD, cD = 5, 3, 4, 6, 2
    x = rng.normal(size=(B, F * N))
    Wp, bp = rng.normal(size=(pD, F * N)), rng.normal(size=pD)
    Wf, bf = rng.normal(size=(cD, N)), rng.normal(size=cD)
    y = oracle.tm_dlrm(x, F, Wp, bp, Wf, bf)
    assert y.shape == (B, pD + F * cD)                       # O = D (c |F| + p)
    assert np.allclose(y[:, :pD], x @ Wp.T + bp, rtol=0, atol=1e-12)
    o2 = np.einsum("bfn,jn->bfj", x.reshape(B, F, N), Wf) + bf
    assert np.allclose(y[:, pD:], o2.reshape(B, F * cD), rtol=0, atol=1e-12)
    # without the per-feature branch (c = 0) it is the plain linear module
    y0 = oracle.tm_dlrm(x, F, Wp, bp, np.zeros((0, N)), np.zeros(0))
    assert np.array_equal(y0, oracle.tm_linear(x, Wp, bp))


def test_lowrank_cross_module_equals_the_full_rank_one_with_the_product_matrix():
    # U (V x) = (U V) x: the low-rank module is the full-rank module with W_l = U_l V_l
    rng = np.random.default_rng(12)
    B, d, r, O = 6, 5, 2, 3
    x = rng.normal(size=(B, d))
    Vc = [0.4 * rng.normal(size=(r, d)) for _ in range(2)]
    Uc = [0.4 * rng.normal(size=(d, r)) for _ in range(2)]
    bc = [rng.normal(size=d) for _ in range(2)]
    W, b = rng.normal(size=(O, d)), rng.normal(size=O)
    y = oracle.tm_cross_lowrank_linear(x, Vc, Uc, bc, W, b)
    full = oracle.tm_cross_linear(x, [U @ V for U, V in zip(Uc, Vc)], bc, W, b)
    assert np.allclose(y, full, rtol=0, atol=1e-12)
    # scalar by hand: d = r = 1, x = 2, v = 3, u = 0.5, c = 1: x1 = 2 * (0.5 * 3 * 2 + 1) + 2 = 10; y = 5 * 10
    y = oracle.tm_cross_lowrank_linear([[2.0]], [[[3.0]]], [[[0.5]]], [[1.0]], [[5.0]], [0.0])
    assert y.tolist() == [[50.0]]
