"""Python face of the CPU oracle (oracle/dmt_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package; the product package never does.  It marshals numpy arrays into
the C loops and rounds the double results once to the requested storage type.
Nothing here touches the HIP library.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import List, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "dmt_oracle.c")
_LIB = os.path.join(_HERE, "libdmt_oracle.so")

DT = {"f32": 0, "f16": 1, "bf16": 2}


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (-O2, OpenMP).  DMT_ORACLE_LIB names a library built
    elsewhere from the same source instead (the sanitizer test's -fsanitize build)."""
    if os.environ.get("DMT_ORACLE_LIB"):
        return os.environ["DMT_ORACLE_LIB"]
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-ffp-contract=off", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_threads.restype = ctypes.c_int
        _lib.oracle_unique.restype = ctypes.c_int64
        _lib.oracle_bwd_accumulate.restype = ctypes.c_int64
        _lib.oracle_sort_keys.restype = ctypes.c_int
    return _lib


def threads() -> int:
    return int(lib().oracle_threads())


def set_threads(n: int) -> None:
    lib().oracle_set_threads(ctypes.c_int(n))


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _i32(x) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.int32)


def _i64(x) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.int64)


def _f64(x) -> np.ndarray:
    return np.ascontiguousarray(x, dtype=np.float64)


def _ptr_array(arrs: Sequence[np.ndarray]):
    return (ctypes.c_void_p * len(arrs))(*[a.ctypes.data for a in arrs])


def decode(a: np.ndarray, dtype: str) -> np.ndarray:
    """Stored elements (float32 / float16 / bfloat16 bits as uint16) -> float64."""
    a = np.ascontiguousarray(a)
    out = np.empty(a.shape, dtype=np.float64)
    lib().oracle_decode(_p(a), DT[dtype], ctypes.c_int64(a.size), _p(out))
    return out


def round_to(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float64 once, to nearest even, into the storage type.  Returns the
    storage array (uint16 bit patterns for bf16)."""
    x = _f64(x)
    if dtype == "f32":
        return x.astype(np.float32)
    if dtype == "f16":
        return x.astype(np.float16)
    # bfloat16 straight from the double: keep 8 significand bits.
    u = x.view(np.uint64)
    sign = (u >> np.uint64(63)).astype(np.uint16) << np.uint16(15)
    ax = np.abs(x)
    out = np.zeros(x.shape, dtype=np.uint16)
    fin = np.isfinite(ax) & (ax > 0)
    m, e = np.frexp(np.where(fin, ax, 1.0))           # ax = m * 2^e, m in [0.5, 1)
    be = e - 1 + 127                                   # biased exponent of 1.f form
    normal = be >= 1
    # normal: 8 significant bits; subnormal: spacing 2^-133
    scale = np.where(normal, 8 - e, 133).astype(np.int64)
    q = np.rint(np.ldexp(np.where(fin, ax, 0.0), scale))     # rint = ties to even
    # normal: q in [128, 256]; bits = (be << 7) + (q - 128) also handles q == 256
    bits = np.where(normal, (be.astype(np.int64) << 7) + (q.astype(np.int64) - 128),
                    q.astype(np.int64))
    bits = np.where(bits >= 0x7F80, 0x7F80, bits)      # overflow -> inf
    out = np.where(fin, bits, 0).astype(np.uint16)
    out = np.where(np.isinf(ax), np.uint16(0x7F80), out)
    out = np.where(np.isnan(x), np.uint16(0x7FC0), out)
    return (out | sign).astype(np.uint16)


def lookup_global(tables: Sequence[np.ndarray], dtype: str, dims, indices, offsets,
                  B: int) -> np.ndarray:
    """Untowered pooled lookup, float64 [B, sum(dims)], features in table order."""
    F = len(tables)
    tables = [np.ascontiguousarray(t) for t in tables]
    dims, indices, offsets = _i32(dims), _i32(indices), _i64(offsets)
    out = np.empty((B, int(dims.sum())), dtype=np.float64)
    lib().oracle_lookup_global(F, _p(dims), DT[dtype], _ptr_array(tables), _p(indices),
                               _p(offsets), ctypes.c_int64(B), _p(out))
    return out


def lookup_towered(tables: Sequence[np.ndarray], dtype: str, dims, table_to_tower,
                   indices, offsets, B: int) -> List[np.ndarray]:
    """Towered pooled lookup: list over towers of float64 [B, W_t] (views of one
    tower-major buffer, also returned flat as the last element's .base)."""
    F = len(tables)
    tables = [np.ascontiguousarray(t) for t in tables]
    dims, t2t = _i32(dims), _i32(table_to_tower)
    indices, offsets = _i32(indices), _i64(offsets)
    T = int(t2t.max()) + 1
    widths = [int(dims[t2t == t].sum()) for t in range(T)]
    flat = np.empty(B * sum(widths), dtype=np.float64)
    lib().oracle_lookup_towered(F, _p(dims), DT[dtype], _ptr_array(tables), T, _p(t2t),
                                _p(indices), _p(offsets), ctypes.c_int64(B), _p(flat))
    out, base = [], 0
    for w in widths:
        out.append(flat[base:base + B * w].reshape(B, w))
        base += B * w
    return out


def tm_linear(x, W, b, relu: bool = False) -> np.ndarray:
    x, W, b = _f64(x), _f64(W), _f64(b)
    B, kin = x.shape
    out = W.shape[0]
    assert W.shape == (out, kin) and b.shape == (out,)
    y = np.empty((B, out), dtype=np.float64)
    lib().oracle_tm_linear(ctypes.c_int64(B), kin, out, _p(x), _p(W), _p(b), int(relu), _p(y))
    return y


def tm_dot_linear(x, nf: int, W, b, return_z: bool = False):
    """x: [B, nf*n]; W: [out, nf(nf-1)/2 + nf*n]."""
    x, W, b = _f64(x), _f64(W), _f64(b)
    B, wt = x.shape
    n = wt // nf
    assert nf * n == wt
    kin = nf * (nf - 1) // 2 + wt
    out = W.shape[0]
    assert W.shape == (out, kin) and b.shape == (out,)
    z = np.empty((B, kin), dtype=np.float64)
    y = np.empty((B, out), dtype=np.float64)
    lib().oracle_tm_dot_linear(ctypes.c_int64(B), nf, n, out, _p(x), _p(W), _p(b), _p(z), _p(y))
    return (y, z) if return_z else y


def tm_dlrm(x, nf: int, Wp, bp, Wf, bf) -> np.ndarray:
    """The DLRM Tower Module (paper Sec. 4, Listing 1) on x [B, nf*n] = embs (B, |F|, N) flattened:
    o1 = the flat embeddings through one Linear(N|F| -> pD); o2 = every feature's embedding
    through ONE shared Linear(N -> cD); result = [o1 | o2 of feature 0 | o2 of feature 1 | ...],
    O = pD + |F| cD columns.  Wp [pD, nf*n], Wf [cD, n]."""
    x, Wp, bp, Wf, bf = _f64(x), _f64(Wp), _f64(bp), _f64(Wf), _f64(bf)
    B, wt = x.shape
    n = wt // nf
    assert nf * n == wt and Wf.shape[1] == n
    parts = [tm_linear(x, Wp, bp)]
    for f in range(nf):
        parts.append(tm_linear(x[:, f * n:(f + 1) * n], Wf, bf))
    return np.concatenate(parts, axis=1)


def cross_layer(x0, x, W, b) -> np.ndarray:
    x0, x, W, b = _f64(x0), _f64(x), _f64(W), _f64(b)
    B, d = x.shape
    assert x0.shape == (B, d) and W.shape == (d, d) and b.shape == (d,)
    xn = np.empty((B, d), dtype=np.float64)
    lib().oracle_cross_layer(ctypes.c_int64(B), d, _p(x0), _p(x), _p(W), _p(b), _p(xn))
    return xn


def tm_cross_linear(x, Wc, bc, W, b) -> np.ndarray:
    """x_{l+1} = x0 * (W_l x_l + b_l) + x_l for every cross layer, then Linear."""
    x0 = _f64(x)
    xl = x0
    for Wl, bl in zip(Wc, bc):
        xl = cross_layer(x0, xl, Wl, bl)
    return tm_linear(xl, W, b)


def tm_cross_lowrank_linear(x, Vc, Uc, bc, W, b) -> np.ndarray:
    """The DCN Tower Module (paper Sec. 4, Listing 2) with low-rank cross layers, the DCN-v2
    form whose d x d matrix is the product of a d x r and an r x d factor:
    x_{l+1} = x0 * (U_l (V_l x_l) + b_l) + x_l with V_l [r, d], U_l [d, r]; then Linear."""
    x0 = _f64(x)
    xl = x0
    for Vl, Ul, bl in zip(Vc, Uc, bc):
        Vl, Ul, bl = _f64(Vl), _f64(Ul), _f64(bl)
        t = tm_linear(xl, Vl, np.zeros(Vl.shape[0]))
        u = tm_linear(t, Ul, bl)
        xl = x0 * u + xl
    return tm_linear(xl, W, b)


def sort_keys(F: int, B: int, indices, offsets):
    """Stable sort of all lookups by (table, row).  Returns int64 arrays
    (sorted_table, sorted_row, sorted_pos)."""
    indices, offsets = _i32(indices), _i64(offsets)
    nnz = int(offsets[F * B])
    st, sr, sp = (np.empty(nnz, dtype=np.int64) for _ in range(3))
    rc = lib().oracle_sort_keys(F, ctypes.c_int64(B), _p(indices), _p(offsets),
                                _p(st), _p(sr), _p(sp))
    if rc:
        raise MemoryError
    return st, sr, sp


def unique(sorted_table, sorted_row):
    """Distinct (table, row) pairs of a sorted key list and their run starts:
    (uniq_table [U], uniq_row [U], seg_off [U+1])."""
    st, sr = _i64(sorted_table), _i64(sorted_row)
    n = len(st)
    ut, ur, so = np.empty(n, np.int64), np.empty(n, np.int64), np.empty(n + 1, np.int64)
    U = int(lib().oracle_unique(ctypes.c_int64(n), _p(st), _p(sr), _p(ut), _p(ur), _p(so)))
    return ut[:U].copy(), ur[:U].copy(), so[:U + 1].copy()


def bwd_accumulate(dims, table_to_tower, indices, offsets, B: int, grad):
    """Dictionary accumulation of row gradients.  Returns (key_table, key_row,
    G [n, Dmax]) sorted ascending by (table, row)."""
    dims, t2t = _i32(dims), _i32(table_to_tower)
    indices, offsets = _i32(indices), _i64(offsets)
    grad = np.ascontiguousarray(grad, dtype=np.float32)
    F, T = len(dims), int(t2t.max()) + 1
    nnz = int(offsets[F * B])
    Dmax = int(dims.max())
    kt, kr = np.empty(nnz, np.int64), np.empty(nnz, np.int64)
    G = np.empty((max(nnz, 1), Dmax), dtype=np.float64)
    n = int(lib().oracle_bwd_accumulate(F, _p(dims), T, _p(t2t), _p(indices), _p(offsets),
                                        ctypes.c_int64(B), _p(grad), Dmax, _p(kt), _p(kr), _p(G)))
    if n < 0:
        raise MemoryError
    kt, kr, G = kt[:n], kr[:n], G[:n]
    order = np.lexsort((kr, kt))
    return kt[order], kr[order], G[order]


def rowwise_adagrad(w_rows, state, G, D_of, lr: float, eps: float):
    """Apply one rowwise-Adagrad step to the given rows.  w_rows [n, Dmax] and
    state [n] are float64 inputs; returns updated float64 copies."""
    w, s, G = _f64(w_rows).copy(), _f64(state).copy(), _f64(G)
    D_of = _i32(D_of)
    n, Dmax = w.shape
    assert G.shape == (n, Dmax) and s.shape == (n,) and D_of.shape == (n,)
    lib().oracle_rowwise_adagrad(ctypes.c_int64(n), Dmax, _p(D_of), _p(G),
                                 ctypes.c_double(lr), ctypes.c_double(eps), _p(w), _p(s))
    return w, s


def bwd_update(tables: Sequence[np.ndarray], dtype: str, states: Sequence[np.ndarray], dims,
               table_to_tower, indices, offsets, B: int, grad, lr: float, eps: float):
    """Whole backward on the CPU: accumulate, then one Adagrad step per touched
    row.  Returns dict(key_table, key_row, G, new_rows (float64 [U, Dmax], not yet
    rounded to the table type), new_state (float64 [U]))."""
    dims = _i32(dims)
    kt, kr, G = bwd_accumulate(dims, table_to_tower, indices, offsets, B, grad)
    Dmax = G.shape[1] if len(G) else int(dims.max())
    w = np.zeros((len(kt), Dmax), dtype=np.float64)
    s = np.zeros(len(kt), dtype=np.float64)
    for f in range(len(tables)):
        m = kt == f
        if not m.any():
            continue
        w[m, :dims[f]] = decode(np.ascontiguousarray(tables[f])[kr[m]], dtype)
        s[m] = np.asarray(states[f], dtype=np.float64)[kr[m]]
    D_of = dims[kt]
    w2, s2 = rowwise_adagrad(w, s, G, D_of, lr, eps)
    return dict(key_table=kt, key_row=kr, G=G, new_rows=w2, new_state=s2, D_of=D_of)
