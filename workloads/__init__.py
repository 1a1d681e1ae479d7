"""Seeded synthetic inputs for the DMT tower hot path.

This module only *draws inputs* (table shapes, tower assignments, jagged id
batches, table values, output gradients, Tower-Module weights).  It holds none
of the method's arithmetic: no pooling, no interaction, no sorting, no
optimizer.  Both the CPU oracle's tests and the HIP path's tests / benchmark
take their inputs from here, and neither of those two imports the other.

The workloads stand in for the paper's: the paper measured throughput on a
random dataset (Sec. 5.3) with Criteo-shaped tables (26 features, N = 128,
about 90 GB, local batch 16K; Sec. 5.1-5.2).  The five named configurations
below keep those shapes and add the skew (bounded Zipf ids, Poisson / Pareto
bag lengths) that real id streams have.
"""
from __future__ import annotations

import dataclasses
import math
from typing import List, Optional, Sequence

import numpy as np

# stream ids for numpy.random.default_rng([seed, stream, table])
_S_ROWS, _S_DIMS, _S_LEN, _S_RANK, _S_PERM, _S_TABLE, _S_GRAD, _S_TM, _S_GRAD_TM = range(9)

F32, F16, BF16 = "f32", "f16", "bf16"
ELT_BYTES = {F32: 4, F16: 2, BF16: 2}

TM_LINEAR, TM_LINEAR_RELU, TM_DOT_LINEAR, TM_CROSS_LINEAR, TM_DLRM, TM_CROSS_LOWRANK_LINEAR = (
    "linear", "linear_relu", "dot_linear", "cross_linear", "dlrm", "cross_lowrank_linear")


@dataclasses.dataclass
class Workload:
    """Static description of one configuration (no arrays)."""
    name: str
    seed: int
    rows: List[int]                 # rows per table
    dims: List[int]                 # embedding dim per table
    table_dtype: str                # f32 / f16 / bf16
    table_to_tower: List[int]       # tower id per table; slot = ascending table id
    batch: int
    len_dist: str                   # "uniform" | "poisson" | "pareto"
    len_param: float                # uniform: max; poisson: mean; pareto: shape
    len_cap: int
    zipf_alpha: Optional[float]     # None -> uniform ids
    tm_kind: str
    tm_out: List[int]               # TM output width per tower
    tm_cross_layers: int
    pooled_dtype: str               # dtype the lookup stores / the TM reads
    tm_dtype: str                   # TM weight and output dtype
    backward: bool
    lr: float = 0.01
    eps: float = 1e-8
    table_std: float = 0.01
    tm_feat_out: int = 0            # TM_DLRM: outputs of the shared per-feature layer (c D);
                                    # tm_out[t] = p D + (tables of tower t) * tm_feat_out.
                                    # TM_CROSS_LOWRANK_LINEAR: the rank r of its cross layers

    @property
    def num_tables(self) -> int:
        return len(self.rows)

    @property
    def num_towers(self) -> int:
        return max(self.table_to_tower) + 1

    def tower_tables(self) -> List[List[int]]:
        out = [[] for _ in range(self.num_towers)]
        for f, t in enumerate(self.table_to_tower):
            out[t].append(f)
        return out

    def tower_widths(self) -> List[int]:
        return [sum(self.dims[f] for f in fs) for fs in self.tower_tables()]

    def tm_in_dims(self) -> List[int]:
        """Width of the vector each tower's projection consumes."""
        out = []
        for fs, w in zip(self.tower_tables(), self.tower_widths()):
            if self.tm_kind == TM_DOT_LINEAR:
                nf = len(fs)
                out.append(nf * (nf - 1) // 2 + w)
            else:
                out.append(w)
        return out


def _log_uniform_rows(seed: int, n: int, lo: int, hi: int) -> List[int]:
    rng = np.random.default_rng([seed, _S_ROWS, 0])
    u = rng.uniform(math.log(lo), math.log(hi), size=n)
    return [int(math.floor(math.exp(x))) for x in u]


def _mean_len(w_len_dist: str, param: float, cap: int) -> float:
    if w_len_dist == "uniform":
        return (1 + param) / 2
    if w_len_dist == "poisson":
        return param
    return 2.5


def tiny() -> Workload:
    return Workload(
        name="tiny", seed=0, rows=[1000] * 8, dims=[16] * 8, table_dtype=F32,
        table_to_tower=[0] * 4 + [1] * 4, batch=64, len_dist="uniform",
        len_param=8, len_cap=8, zipf_alpha=None, tm_kind=TM_LINEAR_RELU,
        tm_out=[32, 32], tm_cross_layers=0, pooled_dtype=F32, tm_dtype=F32,
        backward=True)


def mid(backward: bool = False) -> Workload:
    return Workload(
        name="backward" if backward else "mid", seed=3 if backward else 1,
        rows=[1_000_000] * 64, dims=[128] * 64, table_dtype=F16,
        table_to_tower=[f // 8 for f in range(64)], batch=8192,
        len_dist="poisson", len_param=20, len_cap=100, zipf_alpha=1.05,
        tm_kind=TM_DOT_LINEAR, tm_out=[256] * 8, tm_cross_layers=0,
        pooled_dtype=BF16, tm_dtype=BF16, backward=backward)


def large() -> Workload:
    seed = 2
    rows = _log_uniform_rows(seed, 256, 10_000, 10_000_000)
    # towers balanced by rows x pooling cost: every table has the same mean bag
    # length here, so cost is proportional to rows; deal the tables, sorted by
    # descending cost, to 16 towers in snake order (16 tables per tower).
    order = sorted(range(256), key=lambda f: (-rows[f], f))
    t2t = [0] * 256
    for k, f in enumerate(order):
        rnd, pos = divmod(k, 16)
        t2t[f] = pos if rnd % 2 == 0 else 15 - pos
    return Workload(
        name="large", seed=seed, rows=rows, dims=[128] * 256, table_dtype=BF16,
        table_to_tower=t2t, batch=16384, len_dist="poisson", len_param=30,
        len_cap=200, zipf_alpha=1.1, tm_kind=TM_CROSS_LINEAR,
        tm_out=[512] * 16, tm_cross_layers=2, pooled_dtype=BF16, tm_dtype=BF16,
        backward=False)


IMBALANCED_TOWER_SIZES = [3, 4, 5, 6, 8, 10, 11, 12, 14, 15, 20, 20]


def imbalanced() -> Workload:
    seed = 4
    rows = _log_uniform_rows(seed, 128, 100_000, 5_000_000)
    rng = np.random.default_rng([seed, _S_DIMS, 0])
    dims = [int(x) for x in rng.choice([32, 64, 128], size=128)]
    t2t = []
    for t, n in enumerate(IMBALANCED_TOWER_SIZES):
        t2t += [t] * n
    return Workload(
        name="imbalanced", seed=seed, rows=rows, dims=dims, table_dtype=F16,
        table_to_tower=t2t, batch=65536, len_dist="pareto", len_param=1.5,
        len_cap=500, zipf_alpha=1.2, tm_kind=TM_LINEAR, tm_out=[128] * 12,
        tm_cross_layers=0, pooled_dtype=F16, tm_dtype=F16, backward=True)


def mid_dlrm() -> Workload:
    """Mid's tables and lookups under the DLRM Tower Module of Listing 1 with D = 32 (= N / 4),
    c = 1, p = 4: per tower 8 x 32 per-feature outputs next to 128 flat ones."""
    w = mid()
    w.name = "mid_dlrm"
    w.tm_kind = TM_DLRM
    w.tm_feat_out = 32
    w.tm_out = [4 * 32 + 8 * 32] * 8
    return w


def large_lowrank() -> Workload:
    """Large's tables and lookups under the DCN Tower Module with low-rank cross layers of rank
    512 (a quarter of the tower width)."""
    w = large()
    w.name = "large_lowrank"
    w.tm_kind = TM_CROSS_LOWRANK_LINEAR
    w.tm_feat_out = 512
    return w


def by_name(name: str) -> Workload:
    return {"tiny": tiny, "mid": mid, "large": large, "mid_dlrm": mid_dlrm,
            "large_lowrank": large_lowrank,
            "backward": lambda: mid(True), "imbalanced": imbalanced}[name]()


def tp_embeddings(seed: int, B: int, F: int, N: int, groups: int, noise: float = 0.3) -> np.ndarray:
    """Synthetic pooled embeddings (B, F, N), float64, for the Tower Partitioner: feature f belongs
    to the planted group f % groups; per sample every group draws one N(0, 1) direction that its
    features share, and every feature adds independent N(0, noise^2) on top.  Stands in for the
    embeddings of a trained model (features that interact move together)."""
    rng = np.random.default_rng([seed, 0x7470])
    base = rng.standard_normal((B, groups, N))
    return base[:, np.arange(F) % groups, :] + noise * rng.standard_normal((B, F, N))


def tp_start(seed: int, F: int, n: int, T: int):
    """The Tower Partitioner's random draws: start coordinates N(0, 1) of shape (F, n) and the T
    distinct features whose embedded coordinates serve as start centres."""
    rng = np.random.default_rng([seed, 0x7471])
    return rng.standard_normal((F, n)), np.sort(rng.choice(F, T, replace=False))


def scaled(w: Workload, *, max_rows: Optional[int] = None,
           batch: Optional[int] = None, num_tables: Optional[int] = None,
           name: Optional[str] = None) -> Workload:
    """A smaller instance of `w` with the same structure (for parity tests).

    Keeps dtype, dims, length and id distributions, TM form; clips row counts,
    shrinks the batch and optionally keeps only the first `num_tables` tables
    (towers are renumbered densely in order of first appearance).
    """
    rows, dims, t2t = list(w.rows), list(w.dims), list(w.table_to_tower)
    tm_out = list(w.tm_out)
    if num_tables is not None:
        rows, dims, t2t = rows[:num_tables], dims[:num_tables], t2t[:num_tables]
        remap = {}
        for t in t2t:
            remap.setdefault(t, len(remap))
        tm_out = [w.tm_out[t] for t in remap]
        t2t = [remap[t] for t in t2t]
    if max_rows is not None:
        rows = [min(r, max_rows) for r in rows]
    return dataclasses.replace(
        w, name=name or (w.name + "_small"), rows=rows, dims=dims,
        table_to_tower=t2t, tm_out=tm_out,
        batch=batch if batch is not None else w.batch)


# --------------------------------------------------------------------------
# 16-bit encodings (numpy has no bfloat16: 16-bit tables travel as uint16 bits)
# --------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + r) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def encode(x: np.ndarray, dtype: str) -> np.ndarray:
    """float array -> storage array of `dtype` (f32: float32, f16: float16,
    bf16: uint16 bit patterns)."""
    if dtype == F32:
        return np.ascontiguousarray(x, dtype=np.float32)
    if dtype == F16:
        return np.ascontiguousarray(x).astype(np.float16)
    return f32_to_bf16_bits(x)


def decode(a: np.ndarray, dtype: str) -> np.ndarray:
    """storage array -> float64 values."""
    if dtype == BF16:
        return bf16_bits_to_f32(a).astype(np.float64)
    return a.astype(np.float64)


# --------------------------------------------------------------------------
# jagged id batches
# --------------------------------------------------------------------------

def bag_lengths(w: Workload, batch_id: int = 0) -> np.ndarray:
    """int64 [num_tables * batch], feature-major: bag (f, b) at f*batch + b."""
    out = np.empty(w.num_tables * w.batch, dtype=np.int64)
    for f in range(w.num_tables):
        rng = np.random.default_rng([w.seed, _S_LEN, f, batch_id])
        if w.len_dist == "uniform":
            l = rng.integers(1, int(w.len_param) + 1, size=w.batch)
        elif w.len_dist == "poisson":
            l = np.minimum(rng.poisson(w.len_param, size=w.batch), w.len_cap)
        elif w.len_dist == "pareto":
            u = 1.0 - rng.random(w.batch)            # (0, 1]
            l = np.minimum(np.floor(u ** (-1.0 / w.len_param)), w.len_cap)
        else:
            raise ValueError(w.len_dist)
        out[f * w.batch:(f + 1) * w.batch] = l
    return out


class _ZipfTable:
    """Bounded Zipf over ranks 1..rows, rank -> row by a seeded permutation."""

    def __init__(self, w: Workload, f: int):
        rows = w.rows[f]
        k = np.arange(1, rows + 1, dtype=np.float64)
        cdf = np.cumsum(k ** (-w.zipf_alpha))
        cdf /= cdf[-1]
        self.cdf = cdf
        self.perm = np.random.default_rng(
            [w.seed, _S_PERM, f]).permutation(rows).astype(np.int32)

    def draw(self, rng, n):
        r = np.searchsorted(self.cdf, rng.random(n), side="left")
        np.minimum(r, len(self.cdf) - 1, out=r)
        return self.perm[r]


def lookup_batch(w: Workload, batch_id: int = 0, _cache: Optional[dict] = None):
    """One jagged batch: (indices int32 [nnz], offsets int64 [F*B + 1]).

    Feature-major CSR: bag (f, b) covers indices[offsets[f*B+b]:offsets[f*B+b+1]].
    `_cache` (a dict the caller keeps) memoises the per-table Zipf tables across
    batches.
    """
    lens = bag_lengths(w, batch_id)
    offsets = np.zeros(len(lens) + 1, dtype=np.int64)
    np.cumsum(lens, out=offsets[1:])
    indices = np.empty(int(offsets[-1]), dtype=np.int32)
    for f in range(w.num_tables):
        lo, hi = int(offsets[f * w.batch]), int(offsets[(f + 1) * w.batch])
        rng = np.random.default_rng([w.seed, _S_RANK, f, batch_id])
        if w.zipf_alpha is None:
            indices[lo:hi] = rng.integers(0, w.rows[f], size=hi - lo)
        else:
            zt = _cache.get(f) if _cache is not None else None
            if zt is None:
                zt = _ZipfTable(w, f)
                if _cache is not None:
                    _cache[f] = zt
            indices[lo:hi] = zt.draw(rng, hi - lo)
    return indices, offsets


# --------------------------------------------------------------------------
# tables, gradients, TM weights
# --------------------------------------------------------------------------

def table_host(w: Workload, f: int) -> np.ndarray:
    """Table f as a storage array [rows_f, D_f] (see `encode`)."""
    rng = np.random.default_rng([w.seed, _S_TABLE, f])
    x = rng.standard_normal((w.rows[f], w.dims[f]), dtype=np.float32)
    x *= np.float32(w.table_std)
    return encode(x, w.table_dtype)


def tables_host(w: Workload) -> List[np.ndarray]:
    return [table_host(w, f) for f in range(w.num_tables)]


def tables_device(w: Workload, device="cuda"):
    """Tables drawn on the device with torch's generator (for sizes that do not
    fit a host array comfortably).  Returns a list of torch tensors."""
    import torch
    tdt = {F32: torch.float32, F16: torch.float16, BF16: torch.bfloat16}[w.table_dtype]
    g = torch.Generator(device=device)
    out = []
    for f in range(w.num_tables):
        g.manual_seed((w.seed << 20) + f)
        t = torch.empty((w.rows[f], w.dims[f]), dtype=tdt, device=device)
        t.normal_(0.0, w.table_std, generator=g)
        out.append(t)
    return out


def pooled_layout(w: Workload, batch: Optional[int] = None):
    """Element offsets of the tower-major pooled tensor [T][B][W_t].

    Returns (tower_base [T+1], tower_width [T], col_off [F])."""
    B = w.batch if batch is None else batch
    widths = w.tower_widths()
    base = [0]
    for wt in widths:
        base.append(base[-1] + B * wt)
    col = [0] * w.num_tables
    for fs in w.tower_tables():
        c = 0
        for f in fs:
            col[f] = c
            c += w.dims[f]
    return base, widths, col


def grad_pooled(w: Workload, batch_id: int = 0) -> np.ndarray:
    """N(0,1) float32 gradient w.r.t. the pooled lookup output, tower-major flat."""
    base, _, _ = pooled_layout(w)
    rng = np.random.default_rng([w.seed, _S_GRAD, 0, batch_id])
    return rng.standard_normal(base[-1], dtype=np.float32)


def grad_tm_out(w: Workload, batch_id: int = 0) -> np.ndarray:
    """N(0,1) float32 gradient w.r.t. the Tower Modules' outputs, towers one after
    another, each [B][O_t] row-major, flat."""
    rng = np.random.default_rng([w.seed, _S_GRAD_TM, 0, batch_id])
    return rng.standard_normal(w.batch * sum(w.tm_out), dtype=np.float32)


def tm_weights(w: Workload):
    """Per tower: dict(w_proj [out,in], b_proj [out], w_cross [L][d,d], b_cross [L][d])
    as float32 arrays drawn U(-1/sqrt(in), 1/sqrt(in)); the caller encodes them
    to w.tm_dtype."""
    out = []
    widths = w.tower_widths()
    for t, kin in enumerate(w.tm_in_dims()):
        rng = np.random.default_rng([w.seed, _S_TM, t])
        d = widths[t]
        wc, bc = [], []
        for _ in range(w.tm_cross_layers if w.tm_kind == TM_CROSS_LINEAR else 0):
            s = 1.0 / math.sqrt(d)
            wc.append(rng.uniform(-s, s, size=(d, d)).astype(np.float32))
            bc.append(rng.uniform(-s, s, size=d).astype(np.float32))
        for _ in range(w.tm_cross_layers if w.tm_kind == TM_CROSS_LOWRANK_LINEAR else 0):
            # w_cross = [V_0 [r, d], U_0 [d, r], V_1, U_1, ...]; the product U V is scaled like a
            # full-rank layer's matrix
            r = w.tm_feat_out
            s = 1.0 / math.sqrt(d)
            wc.append(rng.uniform(-s, s, size=(r, d)).astype(np.float32) * math.sqrt(3.0))
            wc.append(rng.uniform(-1, 1, size=(d, r)).astype(np.float32) / math.sqrt(r))
            bc.append(rng.uniform(-s, s, size=d).astype(np.float32))
        o_proj = w.tm_out[t]
        if w.tm_kind == TM_DLRM:
            # the shared per-feature layer rides in the w_cross / b_cross slot 0
            nf = len(w.tower_tables()[t])
            n = d // nf
            s = 1.0 / math.sqrt(n)
            wc.append(rng.uniform(-s, s, size=(w.tm_feat_out, n)).astype(np.float32))
            bc.append(rng.uniform(-s, s, size=w.tm_feat_out).astype(np.float32))
            o_proj = w.tm_out[t] - nf * w.tm_feat_out
        s = 1.0 / math.sqrt(kin)
        out.append(dict(
            w_proj=rng.uniform(-s, s, size=(o_proj, kin)).astype(np.float32),
            b_proj=rng.uniform(-s, s, size=o_proj).astype(np.float32),
            w_cross=wc, b_cross=bc))
    return out


# --------------------------------------------------------------------------
# device-side batch generation (torch), for configurations whose id streams are
# too large to draw with numpy in reasonable time (Large: 126 M ids over tables
# of up to 10 M rows; Imbalanced: 8.4 M bags).  Same distributions as above, a
# different (torch) random stream.
# --------------------------------------------------------------------------

def lookup_batch_device(w: Workload, batch_id: int = 0, device="cuda"):
    """(indices int32 [nnz], offsets int64 [F*B + 1]) as device tensors."""
    import torch
    g = torch.Generator(device=device)
    B = w.batch
    lens = []
    for f in range(w.num_tables):
        g.manual_seed(((w.seed * 1000 + batch_id) << 20) + (_S_LEN << 16) + f)
        if w.len_dist == "uniform":
            l = torch.randint(1, int(w.len_param) + 1, (B,), generator=g, device=device)
        elif w.len_dist == "poisson":
            rate = torch.full((B,), float(w.len_param), device=device)
            l = torch.poisson(rate, generator=g).clamp_(max=w.len_cap).to(torch.int64)
        else:
            u = 1.0 - torch.rand(B, generator=g, device=device, dtype=torch.float64)
            l = torch.floor(u ** (-1.0 / w.len_param)).clamp_(max=w.len_cap).to(torch.int64)
        lens.append(l)
    lens = torch.cat(lens)
    offsets = torch.zeros(w.num_tables * B + 1, dtype=torch.int64, device=device)
    torch.cumsum(lens, 0, out=offsets[1:])
    bounds = offsets[::B].cpu().tolist()
    indices = torch.empty(bounds[-1], dtype=torch.int32, device=device)
    for f in range(w.num_tables):
        lo, hi = bounds[f], bounds[f + 1]
        rows = w.rows[f]
        g.manual_seed(((w.seed * 1000 + batch_id) << 20) + (_S_RANK << 16) + f)
        if w.zipf_alpha is None:
            indices[lo:hi] = torch.randint(0, rows, (hi - lo,), generator=g, device=device, dtype=torch.int32)
            continue
        k = torch.arange(1, rows + 1, device=device, dtype=torch.float64)
        cdf = torch.cumsum(k.pow_(-w.zipf_alpha), 0)
        cdf /= cdf[-1].clone()
        u = torch.rand(hi - lo, generator=g, device=device, dtype=torch.float64)
        r = torch.searchsorted(cdf, u).clamp_(max=rows - 1)
        g.manual_seed((w.seed << 20) + (_S_PERM << 16) + f)          # same permutation for every batch
        perm = torch.randperm(rows, generator=g, device=device)
        indices[lo:hi] = perm[r].to(torch.int32)
        del k, cdf, u, r, perm
    return indices, offsets
