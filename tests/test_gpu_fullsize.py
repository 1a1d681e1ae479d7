"""Parity at the benchmark's full size (the Backward workload = Mid tables and
lookups, 64 x 1M x 128 fp16, B = 8192), in the launch configuration bench.py
times.  The oracle cannot redo 10.5 M lookups over 16 GB of tables in seconds,
so it recomputes SAMPLED outputs one by one from the rows they touch, and the
integer stages are checked through properties that hold at any size.

Tables are drawn on the device (torch's seeded generator: inputs, not the
library's work); the oracle sees the rows it needs through a device -> host copy
of those rows taken BEFORE the library runs."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from harness import TORCH_DT, assert_close, to_device, to_f64

pytestmark = pytest.mark.gpu


class FullRun:
    def __init__(self):
        import paper_2403_00877_amd as dmt
        self.dmt = dmt
        w = self.w = wl.by_name("backward")
        F, B = w.num_tables, w.batch
        self.tables = wl.tables_device(w)
        self.states = [torch.zeros(r, dtype=torch.float32, device="cuda") for r in w.rows]
        self.idx, self.off = wl.lookup_batch(w, 0)
        self.grad = wl.grad_pooled(w, 0)
        nnz = len(self.idx)
        self.plan = dmt.dmt_plan_create(w.rows, w.dims, w.table_dtype, w.num_towers, w.table_to_tower, B, nnz)
        dmt.dmt_plan_bind(self.plan, self.tables, self.states)
        self.base, self.widths, self.col = dmt.dmt_plan_layout(self.plan, B)
        rng = np.random.default_rng(123)

        # ---- samples, and the table rows they need, fetched before anything runs
        self.samples = np.sort(rng.choice(B, size=96, replace=False))
        self.tab_of_pos = np.repeat(np.arange(F, dtype=np.int64), np.diff(self.off[::B]))
        key = (self.tab_of_pos << 32) | self.idx
        uk, counts = np.unique(key, return_counts=True)
        self.uk, self.counts = uk, counts
        hot = uk[np.argsort(-counts)[:40]]                      # the longest runs (span many tiles)
        rest = rng.choice(uk, size=1500, replace=False)
        self.row_keys = np.unique(np.concatenate([hot, rest]))
        self.rows_before = {}
        for f in range(F):
            r = self.row_keys[(self.row_keys >> 32) == f] & 0xffffffff
            self.rows_before[f] = (r, self.tables[f][torch.from_numpy(r).cuda()].cpu().numpy())
        self.fwd_rows = {}
        for f in range(F):
            need = []
            for b in self.samples:
                need.append(self.idx[self.off[f * B + b]:self.off[f * B + b + 1]])
            r = np.unique(np.concatenate(need))
            self.fwd_rows[f] = (r, self.tables[f][torch.from_numpy(r).cuda()].cpu().numpy())
        # an untouched row per table, to see that it stays bit-identical
        self.untouched = {}
        for f in range(F):
            touched = uk[(uk >> 32) == f] & 0xffffffff
            cand = np.setdiff1d(rng.integers(0, w.rows[f], size=64), touched)[:8]
            self.untouched[f] = (cand, self.tables[f][torch.from_numpy(cand).cuda()].clone())

        # ---- the library, once, exactly as bench.py calls it
        self.d_idx, self.d_off = torch.from_numpy(self.idx).cuda(), torch.from_numpy(self.off).cuda()
        self.pooled = torch.empty(self.base[-1], dtype=TORCH_DT[w.pooled_dtype], device="cuda")
        dmt.dmt_tower_lookup_fwd(self.plan, self.d_idx, self.d_off, B, self.pooled)
        tmw = wl.tm_weights(w)
        enc = lambda a: wl.encode(a, w.tm_dtype)
        self.tm_dev = [dict(kind=w.tm_kind, out_dim=w.tm_out[t], w_proj=to_device(enc(h["w_proj"]), w.tm_dtype),
                            b_proj=to_device(enc(h["b_proj"]), w.tm_dtype)) for t, h in enumerate(tmw)]
        self.tm_dec = [dict(w=wl.decode(enc(h["w_proj"]), w.tm_dtype), b=wl.decode(enc(h["b_proj"]), w.tm_dtype))
                       for h in tmw]
        params = dmt.make_tm_params(self.tm_dev)
        ws = torch.empty(max(dmt.dmt_tm_workspace_bytes(self.plan, params, B), 256), dtype=torch.uint8, device="cuda")
        self.tm_out = torch.empty(B * sum(w.tm_out), dtype=TORCH_DT[w.tm_dtype], device="cuda")
        dmt.dmt_tower_module_fwd(self.plan, params, self.pooled, B, self.tm_out, ws)
        bws = torch.empty(dmt.dmt_bwd_workspace_bytes(self.plan, B, nnz), dtype=torch.uint8, device="cuda")
        self.dbg = dict(sorted_keys=torch.empty(nnz, dtype=torch.int64, device="cuda"),
                        sorted_bag=torch.empty(nnz, dtype=torch.int32, device="cuda"),
                        unique_keys=torch.empty(nnz, dtype=torch.int64, device="cuda"),
                        seg_off=torch.empty(nnz + 1, dtype=torch.int64, device="cuda"),
                        num_unique=torch.zeros(1, dtype=torch.int64, device="cuda"))
        dmt.dmt_tower_lookup_bwd_update(self.plan, self.d_idx, self.d_off, B, torch.from_numpy(self.grad).cuda(),
                                        w.lr, w.eps, bws, debug=self.dbg)
        torch.cuda.synchronize()
        assert dmt.dmt_last_device_error(self.plan) == -1


@pytest.fixture(scope="module")
def run():
    r = FullRun()
    yield r
    del r
    torch.cuda.empty_cache()


def _compact(rows_by_table, F, dims, dtype):
    """Small stand-in tables holding only the fetched rows, plus id remaps."""
    tabs, remap = [], []
    for f in range(F):
        r, vals = rows_by_table[f]
        if len(r) == 0:
            vals = np.zeros((1, dims[f]), dtype=vals.dtype)
        tabs.append(np.ascontiguousarray(vals))
        remap.append(r)
    return tabs, remap


def test_lookup_and_tower_module_on_sampled_samples(run):
    w = run.w
    F, B, S = w.num_tables, w.batch, len(run.samples)
    tabs, remap = _compact(run.fwd_rows, F, w.dims, w.table_dtype)
    lens, ids = [], []
    for f in range(F):
        for b in run.samples:
            seg = run.idx[run.off[f * B + b]:run.off[f * B + b + 1]]
            lens.append(len(seg))
            ids.append(np.searchsorted(remap[f], seg))
    s_off = np.concatenate([[0], np.cumsum(lens)])
    s_idx = np.concatenate(ids).astype(np.int32)
    ref = oracle.lookup_towered(tabs, w.table_dtype, w.dims, w.table_to_tower, s_idx, s_off, S)
    sel = torch.from_numpy(run.samples).cuda()
    pos = ypos = 0
    for t, wt in enumerate(run.widths):
        got = to_f64(run.pooled[pos:pos + B * wt].reshape(B, wt)[sel])
        x = wl.decode(oracle.round_to(ref[t], w.pooled_dtype), w.pooled_dtype)
        assert_close(got, x, 2e-2, "pooled tower %d" % t)
        y = oracle.tm_dot_linear(x, len(w.tower_tables()[t]), run.tm_dec[t]["w"], run.tm_dec[t]["b"])
        goty = to_f64(run.tm_out[ypos:ypos + B * w.tm_out[t]].reshape(B, -1)[sel])
        assert_close(goty, wl.decode(oracle.round_to(y, w.tm_dtype), w.tm_dtype), 2e-2, "TM tower %d" % t)
        pos += B * wt
        ypos += B * w.tm_out[t]


def test_sort_and_dedup_properties(run):
    w = run.w
    F, B = w.num_tables, w.batch
    nnz = len(run.idx)
    sk = run.dbg["sorted_keys"].cpu().numpy()
    sb = run.dbg["sorted_bag"].cpu().numpy().astype(np.int64)
    # ascending keys; equal keys in ascending bag order (what a stable sort of bag-ordered input gives)
    dk = np.diff(sk)
    assert (dk >= 0).all()
    assert (np.diff(sb)[dk == 0] >= 0).all()
    # a permutation of the input: same multiset of (key, bag) pairs
    bag_of_pos = np.repeat(np.arange(F * B, dtype=np.int64), np.diff(run.off))
    key = (run.tab_of_pos << 32) | run.idx
    a = np.stack([key, bag_of_pos], 1)
    order = np.lexsort((bag_of_pos, key))
    assert np.array_equal(np.stack([sk, sb], 1), a[order])
    # dedup: numpy.unique on the raw keys
    U = int(run.dbg["num_unique"].item())
    assert U == len(run.uk)
    assert np.array_equal(run.dbg["unique_keys"].cpu().numpy()[:U], run.uk)
    so = run.dbg["seg_off"].cpu().numpy()[:U + 1]
    assert np.array_equal(so, np.concatenate([[0], np.cumsum(run.counts)]))


def test_sampled_row_updates(run):
    """Rowwise-Adagrad results of 1500 random rows and the 40 hottest rows (their
    runs cross many reduce tiles), recomputed by the oracle from those rows' own
    lookups."""
    w = run.w
    F, B = w.num_tables, w.batch
    key = (run.tab_of_pos << 32) | run.idx
    keep = np.isin(key, run.row_keys)
    bag_of_pos = np.repeat(np.arange(F * B, dtype=np.int64), np.diff(run.off))
    tabs, remap = _compact(run.rows_before, F, w.dims, w.table_dtype)
    k_idx = run.idx[keep]
    k_tab = run.tab_of_pos[keep]
    new_idx = np.empty(len(k_idx), dtype=np.int32)
    for f in range(F):
        m = k_tab == f
        new_idx[m] = np.searchsorted(remap[f], k_idx[m])
    new_off = np.concatenate([[0], np.cumsum(np.bincount(bag_of_pos[keep], minlength=F * B))])
    states = [np.zeros(max(len(remap[f]), 1), dtype=np.float32) for f in range(F)]
    ref = oracle.bwd_update(tabs, w.table_dtype, states, w.dims, w.table_to_tower, new_idx, new_off, B,
                            run.grad, w.lr, w.eps)
    assert len(ref["key_row"]) == len(run.row_keys)
    for f in range(F):
        m = ref["key_table"] == f
        if not m.any():
            continue
        real_rows = remap[f][ref["key_row"][m]]
        sel = torch.from_numpy(real_rows).cuda()
        want = wl.decode(oracle.round_to(ref["new_rows"][m][:, :w.dims[f]], w.table_dtype), w.table_dtype)
        assert_close(to_f64(run.tables[f][sel]), want, 2e-2, "rows of table %d" % f)
        assert_close(to_f64(run.states[f][sel]), ref["new_state"][m], 1e-5, "state of table %d" % f)
        # and to the last bit of the table dtype for nearly all elements: float32 vs float64 can only
        # differ where the exact result sits on a rounding boundary
        got_bits = run.tables[f][sel].view(torch.int16).cpu().numpy()
        want_bits = oracle.round_to(ref["new_rows"][m][:, :w.dims[f]], w.table_dtype).view(np.int16)
        assert (np.abs(got_bits.astype(np.int32) - want_bits.astype(np.int32)) <= 1).mean() > 0.999


def test_untouched_rows_and_states_are_bit_identical(run):
    for f, (cand, before) in run.untouched.items():
        sel = torch.from_numpy(cand).cuda()
        assert torch.equal(run.tables[f][sel].view(torch.int16), before.view(torch.int16))
        assert torch.count_nonzero(run.states[f][sel]).item() == 0
    # the number of rows with a non-zero state is exactly the number of distinct rows touched
    touched = sum(int(torch.count_nonzero(s).item()) for s in run.states)
    assert touched == len(run.uk)
