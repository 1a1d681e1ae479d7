"""Row-wise sharded tables (paper Sec. 3.1.3) on the GPU against the oracle: every shard pools
and updates the rows it holds, from the unchanged ids of the whole table; the partial pools add
up to the lookup, and the shards' updated rows are the unsharded update's rows."""
import numpy as np
import pytest
import torch

import oracle
import paper_2403_00877_amd as dmt
import workloads as wl
from harness import RTOL, assert_close, to_device, to_f64
from oracle import sptt

pytestmark = pytest.mark.gpu


def _cuts(w, nshards, rng):
    """Per table, the first row of each shard (+ the row count at the end); shards may be empty."""
    cuts = []
    for r in w.rows:
        inner = np.sort(rng.integers(0, r + 1, size=nshards - 1))
        cuts.append([0] + [int(x) for x in inner] + [r])
    return cuts


class Shard:
    def __init__(self, w, host_tables, lo, n, with_state, max_nnz):
        F = w.num_tables
        self.lo, self.n = lo, n
        # a plan needs at least one row per table: an empty shard holds one row nobody looks up
        self.rows = [max(1, k) for k in n]
        self.host = [host_tables[f][lo[f]:lo[f] + n[f]] if n[f] else np.zeros_like(host_tables[f][:1])
                     for f in range(F)]
        self.tables = [to_device(t, w.table_dtype) for t in self.host]
        self.states = [torch.zeros(r, dtype=torch.float32, device="cuda") for r in self.rows] if with_state else None
        self.plan = dmt.dmt_plan_create(self.rows, w.dims, w.table_dtype, w.num_towers, w.table_to_tower,
                                        w.batch, max_nnz)
        # an empty shard's stand-in row sits past every id of the table
        begin = [lo[f] if n[f] else 2 ** 31 - 1 for f in range(F)]
        dmt.dmt_plan_set_row_shards(self.plan, begin)
        dmt.dmt_plan_bind(self.plan, self.tables, self.states)


@pytest.mark.parametrize("name,nshards", [("tiny", 2), ("mid", 3), ("imbalanced", 4)])
def test_partial_pools_match_the_oracle_and_add_up(name, nshards):
    w = {"tiny": wl.tiny(),
         "mid": wl.scaled(wl.mid(), max_rows=3000, batch=203, num_tables=16),
         "imbalanced": wl.scaled(wl.imbalanced(), max_rows=2000, batch=333, num_tables=12)}[name]
    _check_partial_pools(w, nshards, np.random.default_rng(5), name)


def _check_partial_pools(w, nshards, rng, name):
    F, B = w.num_tables, w.batch
    host = wl.tables_host(w)
    idx, off = wl.lookup_batch(w)
    d_idx, d_off = torch.from_numpy(idx).cuda(), torch.from_numpy(off).cuda()
    base, widths, col = wl.pooled_layout(w)
    full = oracle.lookup_towered(host, w.table_dtype, w.dims, w.table_to_tower, idx, off, B)
    cuts = _cuts(w, nshards, rng)
    total = torch.zeros(base[-1], dtype=torch.float32, device="cuda")
    for s in range(nshards):
        lo = [cuts[f][s] for f in range(F)]
        n = [cuts[f][s + 1] - cuts[f][s] for f in range(F)]
        sh = Shard(w, host, lo, n, False, len(idx))
        out = torch.full((base[-1],), float("nan"), dtype=torch.float32, device="cuda")
        dmt.dmt_tower_lookup_fwd(sh.plan, d_idx, d_off, B, out)       # the whole table's ids, unchanged
        torch.cuda.synchronize()
        assert dmt.dmt_last_device_error(sh.plan) == -1               # other shards' ids are no error
        s_idx, s_off = sptt.row_shard_lookups(idx, off, F, B, lo, n)
        ref = oracle.lookup_towered(sh.host, w.table_dtype, w.dims, w.table_to_tower, s_idx, s_off, B)
        got = to_f64(out)
        for t in range(w.num_towers):
            assert_close(got[base[t]:base[t + 1]].reshape(B, widths[t]), ref[t], 1e-5,
                         "%s shard %d tower %d" % (name, s, t))
        total += out                                                  # the ReduceScatter's sum
    got = to_f64(total)
    for t in range(w.num_towers):
        assert_close(got[base[t]:base[t + 1]].reshape(B, widths[t]), full[t], 1e-5, "%s sum of shards" % name)


@pytest.mark.parametrize("name,nshards", [("tiny", 2), ("mid", 3)])
def test_sharded_update_is_the_unsharded_update_row_by_row(name, nshards):
    w = {"tiny": wl.tiny(),
         "mid": wl.scaled(wl.mid(True), max_rows=4000, batch=203, num_tables=16)}[name]
    _check_sharded_update(w, nshards, np.random.default_rng(6), name)


@pytest.mark.parametrize("seed", range(12))
def test_random_configurations_in_random_shards(seed):
    """Arbitrary table sets cut into 2 to 4 uneven row shards (some empty)."""
    from test_gpu_random_shapes import random_workload
    w = random_workload(1500 + seed)
    if len(wl.lookup_batch(w)[0]) == 0:
        pytest.skip("no lookups drawn")
    nshards = 2 + seed % 3
    _check_partial_pools(w, nshards, np.random.default_rng([7, seed]), w.name)
    _check_sharded_update(w, nshards, np.random.default_rng([8, seed]), w.name)


def _check_sharded_update(w, nshards, rng, name):
    F, B = w.num_tables, w.batch
    host = wl.tables_host(w)
    idx, off = wl.lookup_batch(w)
    grad = wl.grad_pooled(w)
    d_idx, d_off, d_grad = torch.from_numpy(idx).cuda(), torch.from_numpy(off).cuda(), torch.from_numpy(grad).cuda()
    st0 = [np.zeros(r, dtype=np.float32) for r in w.rows]
    ref = oracle.bwd_update(host, w.table_dtype, st0, w.dims, w.table_to_tower, idx, off, B, grad, w.lr, w.eps)
    rtol = RTOL[w.table_dtype]
    cuts = _cuts(w, nshards, rng)
    seen = 0
    for s in range(nshards):
        lo = [cuts[f][s] for f in range(F)]
        n = [cuts[f][s + 1] - cuts[f][s] for f in range(F)]
        sh = Shard(w, host, lo, n, True, len(idx))
        before = [t.clone() for t in sh.tables]
        ws = torch.empty(max(dmt.dmt_bwd_workspace_bytes(sh.plan, B, len(idx)), 256), dtype=torch.uint8, device="cuda")
        dmt.dmt_tower_lookup_bwd_update(sh.plan, d_idx, d_off, B, d_grad, w.lr, w.eps, ws)
        torch.cuda.synchronize()
        assert dmt.dmt_last_device_error(sh.plan) == -1
        for f in range(F):
            m = (ref["key_table"] == f) & (ref["key_row"] >= lo[f]) & (ref["key_row"] < lo[f] + n[f])
            local = ref["key_row"][m] - lo[f]
            seen += int(m.sum())
            D = w.dims[f]
            sel = torch.from_numpy(local).cuda()
            want = ref["new_rows"][m][:, :D]
            if w.table_dtype != "f32":
                want = wl.decode(oracle.round_to(want, w.table_dtype), w.table_dtype)
            assert_close(to_f64(sh.tables[f][sel]), want, rtol, "%s shard %d rows of table %d" % (name, s, f))
            assert_close(to_f64(sh.states[f][sel]), ref["new_state"][m].astype(np.float32), 1e-5,
                         "%s shard %d state of table %d" % (name, s, f))
            # local rows that no lookup touched keep their bits
            untouched = np.ones(sh.rows[f], bool)
            untouched[local] = False
            u = torch.from_numpy(np.nonzero(untouched)[0]).cuda()
            bits = torch.int32 if w.table_dtype == "f32" else torch.int16
            assert torch.equal(sh.tables[f][u].view(bits), before[f][u].view(bits))
            assert float(sh.states[f][u].abs().sum()) == 0.0
    assert seen == len(ref["key_row"])          # every touched row lives in exactly one shard


def test_set_row_shards_rejects_bad_arguments():
    w = wl.tiny()
    plan = dmt.dmt_plan_create(w.rows, w.dims, w.table_dtype, w.num_towers, w.table_to_tower, w.batch, 100)
    raw = dmt.binding._lib.dmt_plan_set_row_shards
    import ctypes
    ok = (ctypes.c_int64 * w.num_tables)(*([5] * w.num_tables))
    neg = (ctypes.c_int64 * w.num_tables)(*([-1] * w.num_tables))
    big = (ctypes.c_int64 * w.num_tables)(*([2 ** 31] * w.num_tables))
    assert raw(plan.handle, ok) == 0
    assert raw(None, ok) == 1 and raw(plan.handle, None) == 1
    assert raw(plan.handle, neg) == 1 and raw(plan.handle, big) == 1
