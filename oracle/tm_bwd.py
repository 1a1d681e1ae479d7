"""Backward of the Tower Module forms, CPU oracle.  TEST INFRASTRUCTURE ONLY.

Only tests may import this module; the product package never does, and nothing
here touches the HIP library.

The Tower Module (paper Sec. 3.2, Listings 1 and 2) is a composition of linear
maps, pairwise dot products and DCN-v2 cross layers; its backward is the chain
rule applied to exactly the forward definitions of oracle.tm_linear,
oracle.tm_dot_linear and oracle.tm_cross_linear, written out term by term in
float64 with numpy's matmul as the only library step.  `dy` is dL/dy for some
scalar L; every function returns dL/d(input) and dL/d(parameters).

Pinned in tests/test_oracle_tm_bwd.py against central differences of the
forward oracle (which has pins of its own), closed forms and hand-computed cases.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np


def _f64(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float64)


def tm_linear_bwd(x, W, b, dy, relu: bool = False) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """y = x W^T + b (then max(0, .) if relu).  Returns (dx, dW, db).

    With pre = x W^T + b:  dpre = dy where pre > 0 (all of dy without ReLU);
    dx = dpre W,  dW = dpre^T x,  db = sum over the batch of dpre.
    """
    x, W, b, dy = _f64(x), _f64(W), _f64(b), _f64(dy)
    dpre = dy
    if relu:
        pre = x @ W.T + b
        dpre = dy * (pre > 0)
    return dpre @ W, dpre.T @ x, dpre.sum(axis=0)


def tm_dot_linear_bwd(x, nf: int, W, b, dy) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """z = [p | x] with p[(i,j)] = <x_i, x_j> for i < j in row-major pair order, y = z W^T + b
    (Listing 1 with its per-feature projections switched off).  Returns (dx, dW, db).

    dz = dy W;  dW = dy^T z;  db = sum_b dy;  the flat part of dz goes to x as it is, and
    every pair term adds dp_ij * x_j to dx_i and dp_ij * x_i to dx_j.
    """
    x, W, b, dy = _f64(x), _f64(W), _f64(b), _f64(dy)
    B, wt = x.shape
    n = wt // nf
    assert nf * n == wt
    npair = nf * (nf - 1) // 2
    X = x.reshape(B, nf, n)
    p = np.empty((B, npair), dtype=np.float64)
    k = 0
    for i in range(nf):
        for j in range(i + 1, nf):
            p[:, k] = np.sum(X[:, i, :] * X[:, j, :], axis=1)
            k += 1
    z = np.concatenate([p, x], axis=1)
    dz = dy @ W
    dW = dy.T @ z
    db = dy.sum(axis=0)
    dX = dz[:, npair:].reshape(B, nf, n).copy()
    k = 0
    for i in range(nf):
        for j in range(i + 1, nf):
            dX[:, i, :] += dz[:, k, None] * X[:, j, :]
            dX[:, j, :] += dz[:, k, None] * X[:, i, :]
            k += 1
    return dX.reshape(B, wt), dW, db


def tm_dlrm_bwd(x, nf: int, Wp, bp, Wf, bf, dy):
    """y = [x Wp^T + bp | x_0 Wf^T + bf | ... | x_{F-1} Wf^T + bf] (Listing 1; x_f the f-th
    feature's n columns of x).  Returns (dx, dWp, dbp, dWf, dbf).

    The flat part is a linear layer of its own; the shared per-feature layer receives the sum
    over features of each feature's linear-layer gradients, and dx is the sum of both paths.
    """
    x, Wp, bp, Wf, bf, dy = _f64(x), _f64(Wp), _f64(bp), _f64(Wf), _f64(bf), _f64(dy)
    B, wt = x.shape
    n = wt // nf
    assert nf * n == wt
    pD, cD = Wp.shape[0], Wf.shape[0]
    assert dy.shape == (B, pD + nf * cD)
    dx, dWp, dbp = tm_linear_bwd(x, Wp, bp, dy[:, :pD])
    dx = dx.copy()
    dWf = np.zeros_like(Wf)
    dbf = np.zeros_like(bf)
    for f in range(nf):
        dyf = dy[:, pD + f * cD:pD + (f + 1) * cD]
        dxf, dW, db = tm_linear_bwd(x[:, f * n:(f + 1) * n], Wf, bf, dyf)
        dx[:, f * n:(f + 1) * n] += dxf
        dWf += dW
        dbf += db
    return dx, dWp, dbp, dWf, dbf


def tm_cross_linear_bwd(x, Wc: Sequence, bc: Sequence, W, b, dy):
    """x_{l+1} = x0 * (W_l x_l + b_l) + x_l for every cross layer (x_0 = x0 = x), y = x_L W^T + b
    (Listing 2; the full-rank DCN-v2 layer).  Returns (dx, [dW_l], [db_l], dW, db).

    With u_l = W_l x_l + b_l, going down from l = L-1:
      du_l = dx_{l+1} * x0;  dx0 += dx_{l+1} * u_l;  dW_l = du_l^T x_l;  db_l = sum_b du_l;
      dx_l = du_l W_l + dx_{l+1};
    and x enters both as x_0 and as x0, so dx = dx_0 + dx0.
    """
    x0 = _f64(x)
    Wc = [_f64(w) for w in Wc]
    bc = [_f64(v) for v in bc]
    W, b, dy = _f64(W), _f64(b), _f64(dy)
    xs: List[np.ndarray] = [x0]
    us: List[np.ndarray] = []
    for Wl, bl in zip(Wc, bc):
        u = xs[-1] @ Wl.T + bl
        us.append(u)
        xs.append(x0 * u + xs[-1])
    dxl = dy @ W
    dW = dy.T @ xs[-1]
    db = dy.sum(axis=0)
    dx0 = np.zeros_like(x0)
    dWc: List[np.ndarray] = [None] * len(Wc)
    dbc: List[np.ndarray] = [None] * len(Wc)
    for l in range(len(Wc) - 1, -1, -1):
        du = dxl * x0
        dx0 += dxl * us[l]
        dWc[l] = du.T @ xs[l]
        dbc[l] = du.sum(axis=0)
        dxl = du @ Wc[l] + dxl
    return dxl + dx0, dWc, dbc, dW, db


def tm_cross_lowrank_linear_bwd(x, Vc: Sequence, Uc: Sequence, bc: Sequence, W, b, dy):
    """x_{l+1} = x0 * (U_l (V_l x_l) + b_l) + x_l, y = x_L W^T + b (Listing 2 with the low-rank
    DCN-v2 layer).  Returns (dx, [dV_l], [dU_l], [db_l], dW, db).

    With t_l = V_l x_l and u_l = U_l t_l + b_l, going down from l = L-1:
      du_l = dx_{l+1} * x0;  dx0 += dx_{l+1} * u_l;  dU_l = du_l^T t_l;  db_l = sum_b du_l;
      dt_l = du_l U_l;  dV_l = dt_l^T x_l;  dx_l = dt_l V_l + dx_{l+1};
    and dx = dx_0 + dx0.
    """
    x0 = _f64(x)
    Vc = [_f64(v) for v in Vc]
    Uc = [_f64(u) for u in Uc]
    bc = [_f64(v) for v in bc]
    W, b, dy = _f64(W), _f64(b), _f64(dy)
    xs: List[np.ndarray] = [x0]
    ts: List[np.ndarray] = []
    us: List[np.ndarray] = []
    for Vl, Ul, bl in zip(Vc, Uc, bc):
        t = xs[-1] @ Vl.T
        u = t @ Ul.T + bl
        ts.append(t)
        us.append(u)
        xs.append(x0 * u + xs[-1])
    dxl = dy @ W
    dW = dy.T @ xs[-1]
    db = dy.sum(axis=0)
    dx0 = np.zeros_like(x0)
    L = len(Vc)
    dVc: List[np.ndarray] = [None] * L
    dUc: List[np.ndarray] = [None] * L
    dbc: List[np.ndarray] = [None] * L
    for l in range(L - 1, -1, -1):
        du = dxl * x0
        dx0 += dxl * us[l]
        dUc[l] = du.T @ ts[l]
        dbc[l] = du.sum(axis=0)
        dt = du @ Uc[l]
        dVc[l] = dt.T @ xs[l]
        dxl = dt @ Vc[l] + dxl
    return dxl + dx0, dVc, dUc, dbc, dW, db
