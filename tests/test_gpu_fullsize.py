"""Parity at the benchmark configurations' full sizes, in the launch configurations bench.py
times: Mid under its own seed (forward only), the Backward workload (= Mid tables and
lookups, 64 x 1M x 128 fp16, B = 8192; the benchmark's own step), Imbalanced (128 mixed-width tables,
B = 65536, forward + backward) and Large (256 bf16 tables, ~97 GB, B = 16384,
forward + two cross layers + projection).

The oracle cannot redo 10-126 M lookups over 16-97 GB of tables in seconds, so
it recomputes SAMPLED outputs one by one from the rows they touch, and the
integer stages are checked through properties that hold at any size.

Tables are drawn on the device (torch's seeded generator: inputs, not the
library's work), ids on the host (Backward) or the device (the other two); the
oracle sees the rows it needs through a device -> host copy of those rows taken
BEFORE the library runs."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from oracle import tm_bwd
from harness import TORCH_DT, assert_close, assert_grad_close, oracle_tm, tm_device_and_decoded, to_f64

pytestmark = pytest.mark.gpu

BITS = {"f32": torch.int32, "f16": torch.int16, "bf16": torch.int16}


class FullRun:
    def __init__(self, name, n_samples, n_rows, device_ids):
        import paper_2403_00877_amd as dmt
        self.dmt = dmt
        w = self.w = wl.by_name(name)
        F, B = w.num_tables, w.batch
        self.tables = wl.tables_device(w)
        self.states = ([torch.zeros(r, dtype=torch.float32, device="cuda") for r in w.rows]
                       if w.backward else None)
        if device_ids:
            self.d_idx, self.d_off = wl.lookup_batch_device(w, 0)
            self.idx, self.off = self.d_idx.cpu().numpy(), self.d_off.cpu().numpy()
        else:
            self.idx, self.off = wl.lookup_batch(w, 0)
            self.d_idx, self.d_off = torch.from_numpy(self.idx).cuda(), torch.from_numpy(self.off).cuda()
        nnz = len(self.idx)
        self.plan = dmt.dmt_plan_create(w.rows, w.dims, w.table_dtype, w.num_towers, w.table_to_tower, B, nnz)
        dmt.dmt_plan_bind(self.plan, self.tables, self.states)
        self.base, self.widths, self.col = dmt.dmt_plan_layout(self.plan, B)
        rng = np.random.default_rng(123)

        # ---- samples, and the table rows they need, fetched before anything runs
        self.samples = np.sort(rng.choice(B, size=n_samples, replace=False))
        self.fwd_rows = {}
        for f in range(F):
            need = [self.idx[self.off[f * B + b]:self.off[f * B + b + 1]] for b in self.samples]
            r = np.unique(np.concatenate(need))
            self.fwd_rows[f] = (r, self._fetch(f, r))
        if w.backward:
            g = torch.Generator(device="cuda")
            g.manual_seed(77)
            self.d_grad = torch.randn(self.base[-1], generator=g, device="cuda", dtype=torch.float32)
            self.grad = self.d_grad.cpu().numpy()
            self.tab_of_pos = np.repeat(np.arange(F, dtype=np.int64), np.diff(self.off[::B]))
            key = (self.tab_of_pos << 32) | self.idx
            self.uk, self.counts = np.unique(key, return_counts=True)
            hot = self.uk[np.argsort(-self.counts)[:40]]            # the longest runs (span many tiles)
            rest = rng.choice(self.uk, size=n_rows, replace=False)
            self.row_keys = np.unique(np.concatenate([hot, rest]))
            self.rows_before = {}
            for f in range(F):
                r = self.row_keys[(self.row_keys >> 32) == f] & 0xffffffff
                self.rows_before[f] = (r, self._fetch(f, r))
            # rows no lookup touches, to see that they stay bit-identical
            self.untouched = {}
            for f in range(0, F, max(1, F // 16)):
                touched = self.uk[(self.uk >> 32) == f] & 0xffffffff
                cand = np.setdiff1d(rng.integers(0, w.rows[f], size=64), touched)[:8]
                self.untouched[f] = (cand, self.tables[f][torch.from_numpy(cand).cuda()].clone())

        # ---- the library, once, exactly as bench.py calls it
        self.pooled = torch.empty(self.base[-1], dtype=TORCH_DT[w.pooled_dtype], device="cuda")
        dmt.dmt_tower_lookup_fwd(self.plan, self.d_idx, self.d_off, B, self.pooled)
        tm_dev, self.tm_dec = tm_device_and_decoded(w)
        self._keep = tm_dev
        params = dmt.make_tm_params(tm_dev)
        ws = torch.empty(max(dmt.dmt_tm_workspace_bytes(self.plan, params, B), 256), dtype=torch.uint8, device="cuda")
        self.tm_out = torch.empty(B * sum(w.tm_out), dtype=TORCH_DT[w.tm_dtype], device="cuda")
        dmt.dmt_tower_module_fwd(self.plan, params, self.pooled, B, self.tm_out, ws)
        del ws
        if w.backward:
            bws = torch.empty(dmt.dmt_bwd_workspace_bytes(self.plan, B, nnz), dtype=torch.uint8, device="cuda")
            self.dbg = dict(sorted_keys=torch.empty(nnz, dtype=torch.int64, device="cuda"),
                            sorted_bag=torch.empty(nnz, dtype=torch.int32, device="cuda"),
                            unique_keys=torch.empty(nnz, dtype=torch.int64, device="cuda"),
                            seg_off=torch.empty(nnz + 1, dtype=torch.int64, device="cuda"),
                            num_unique=torch.zeros(1, dtype=torch.int64, device="cuda"))
            dmt.dmt_tower_lookup_bwd_update(self.plan, self.d_idx, self.d_off, B, self.d_grad,
                                            w.lr, w.eps, bws, debug=self.dbg)
            del bws
        torch.cuda.synchronize()
        assert dmt.dmt_last_device_error(self.plan) == -1

    def _fetch(self, f, rows):
        t = self.tables[f][torch.from_numpy(rows).cuda()]
        if self.w.table_dtype == "bf16":
            return t.view(torch.int16).cpu().numpy().view(np.uint16)
        return t.cpu().numpy()


RUNS = {"mid": dict(n_samples=48, n_rows=0, device_ids=False),
        "backward": dict(n_samples=96, n_rows=1500, device_ids=False),
        "imbalanced": dict(n_samples=64, n_rows=1500, device_ids=True),
        "large": dict(n_samples=24, n_rows=0, device_ids=True)}


@pytest.fixture(scope="module", params=list(RUNS))
def run(request):
    r = FullRun(request.param, **RUNS[request.param])
    yield r
    del r
    torch.cuda.empty_cache()


def _compact(rows_by_table, w):
    """Small stand-in tables holding only the fetched rows, plus id remaps."""
    tabs, remap = [], []
    for f in range(w.num_tables):
        r, vals = rows_by_table[f]
        if len(r) == 0:
            vals = np.zeros((1, w.dims[f]), dtype=vals.dtype)
        tabs.append(np.ascontiguousarray(vals))
        remap.append(r)
    return tabs, remap


def _sampled_pooled(run):
    """The oracle's pooled values of the sampled samples, per tower [S][W_t], from the table rows
    fetched before the library ran."""
    w = run.w
    F, B, S = w.num_tables, w.batch, len(run.samples)
    tabs, remap = _compact(run.fwd_rows, w)
    lens, ids = [], []
    for f in range(F):
        for b in run.samples:
            seg = run.idx[run.off[f * B + b]:run.off[f * B + b + 1]]
            lens.append(len(seg))
            ids.append(np.searchsorted(remap[f], seg))
    s_off = np.concatenate([[0], np.cumsum(lens)])
    s_idx = np.concatenate(ids).astype(np.int32)
    return oracle.lookup_towered(tabs, w.table_dtype, w.dims, w.table_to_tower, s_idx, s_off, S)


def test_lookup_and_tower_module_on_sampled_samples(run):
    w = run.w
    B = w.batch
    ref = _sampled_pooled(run)
    sel = torch.from_numpy(run.samples).cuda()
    x = [wl.decode(oracle.round_to(r, w.pooled_dtype), w.pooled_dtype) for r in ref]
    y = oracle_tm(w, run.tm_dec, x)
    pos = ypos = 0
    for t, wt in enumerate(run.widths):
        got = to_f64(run.pooled[pos:pos + B * wt].reshape(B, wt)[sel])
        assert_close(got, x[t], 2e-2, "%s pooled tower %d" % (w.name, t))
        goty = to_f64(run.tm_out[ypos:ypos + B * w.tm_out[t]].reshape(B, -1)[sel])
        assert_close(goty, wl.decode(oracle.round_to(y[t], w.tm_dtype), w.tm_dtype), 2e-2,
                     "%s TM tower %d" % (w.name, t))
        pos += B * wt
        ypos += B * w.tm_out[t]


def test_sort_and_dedup_properties(run):
    w = run.w
    if not w.backward:
        pytest.skip("%s is a forward-only configuration" % w.name)
    F, B = w.num_tables, w.batch
    sk = run.dbg["sorted_keys"].cpu().numpy()
    sb = run.dbg["sorted_bag"].cpu().numpy().astype(np.int64)
    # ascending keys; equal keys in ascending bag order (what a stable sort of bag-ordered input gives)
    dk = np.diff(sk)
    assert (dk >= 0).all()
    assert (np.diff(sb)[dk == 0] >= 0).all()
    # a permutation of the input: same multiset of (key, bag) pairs
    bag_of_pos = np.repeat(np.arange(F * B, dtype=np.int64), np.diff(run.off))
    key = (run.tab_of_pos << 32) | run.idx
    order = np.lexsort((bag_of_pos, key))
    assert np.array_equal(sk, key[order]) and np.array_equal(sb, bag_of_pos[order])
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
    if not w.backward:
        pytest.skip("%s is a forward-only configuration" % w.name)
    F, B = w.num_tables, w.batch
    key = (run.tab_of_pos << 32) | run.idx
    keep = np.isin(key, run.row_keys)
    bag_of_pos = np.repeat(np.arange(F * B, dtype=np.int64), np.diff(run.off))
    tabs, remap = _compact(run.rows_before, w)
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
    near = total = 0
    for f in range(F):
        m = ref["key_table"] == f
        if not m.any():
            continue
        real_rows = remap[f][ref["key_row"][m]]
        sel = torch.from_numpy(real_rows).cuda()
        want_bits = oracle.round_to(ref["new_rows"][m][:, :w.dims[f]], w.table_dtype)
        assert_close(to_f64(run.tables[f][sel]), wl.decode(want_bits, w.table_dtype), 2e-2,
                     "%s rows of table %d" % (w.name, f))
        assert_close(to_f64(run.states[f][sel]), ref["new_state"][m], 1e-5, "state of table %d" % f)
        got_bits = run.tables[f][sel].view(BITS[w.table_dtype]).cpu().numpy()
        near += int((np.abs(got_bits.astype(np.int64) - want_bits.view(got_bits.dtype).astype(np.int64)) <= 1).sum())
        total += got_bits.size
    # and to the last bit of the table dtype for nearly all elements: float32 and float64 can only
    # disagree where the exact result sits on a rounding boundary
    assert near / total > 0.999


def test_untouched_rows_and_states_are_bit_identical(run):
    w = run.w
    if not w.backward:
        pytest.skip("%s is a forward-only configuration" % w.name)
    for f, (cand, before) in run.untouched.items():
        sel = torch.from_numpy(cand).cuda()
        assert torch.equal(run.tables[f][sel].view(BITS[w.table_dtype]), before.view(BITS[w.table_dtype]))
        assert torch.count_nonzero(run.states[f][sel]).item() == 0
    # the number of rows with a non-zero state is exactly the number of distinct rows touched
    touched = sum(int(torch.count_nonzero(s).item()) for s in run.states)
    assert touched == len(run.uk)


def test_tower_module_backward_on_sampled_samples(run):
    """dmt_tower_module_bwd at the full batch, in two calls.  (1) A dense N(0,1) output gradient:
    the input gradient of a sample depends on that sample alone, so the sampled samples' rows
    are compared with the oracle's, and every bias gradient of the projection is the plain
    batch sum of the gradient.  (2) The same gradient kept on the sampled samples only and zero
    elsewhere: now every weight and bias gradient is a sum over the sampled samples, which the
    oracle recomputes in full, and all other samples' input gradients are exactly zero."""
    w = run.w
    dmt = run.dmt
    B, T = w.batch, w.num_towers
    S = len(run.samples)
    nl = w.tm_cross_layers if w.tm_kind == wl.TM_CROSS_LINEAR else 0
    kin, tw = w.tm_in_dims(), w.tower_widths()
    x = [wl.decode(oracle.round_to(r, w.pooled_dtype), w.pooled_dtype) for r in _sampled_pooled(run)]
    params = dmt.make_tm_params(run._keep)
    f32 = lambda *shape: torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    grads = [dict(dw_proj=f32(o, k), db_proj=f32(o), dw_cross=[f32(d, d) for _ in range(nl)],
                  db_cross=[f32(d) for _ in range(nl)]) for o, k, d in zip(w.tm_out, kin, tw)]
    arr = dmt.make_tm_grads(grads)
    ws = torch.empty(dmt.dmt_tm_bwd_workspace_bytes(run.plan, params, B), dtype=torch.uint8, device="cuda")
    g = torch.Generator(device="cuda")
    g.manual_seed(991)
    dy = torch.randn(B * sum(w.tm_out), generator=g, device="cuda", dtype=torch.float32)
    dx = f32(B * sum(tw))
    sel = torch.from_numpy(run.samples).cuda()
    rtol = 4e-2 if nl else 2e-2
    tables_of = w.tower_tables()

    def oracle_bwd(t, dyt):
        d = run.tm_dec[t]
        if w.tm_kind == wl.TM_DOT_LINEAR:
            r = tm_bwd.tm_dot_linear_bwd(x[t], len(tables_of[t]), d["w_proj"], d["b_proj"], dyt)
            return r[0], [], [], r[1], r[2]
        if w.tm_kind == wl.TM_CROSS_LINEAR:
            return tm_bwd.tm_cross_linear_bwd(x[t], d["w_cross"], d["b_cross"], d["w_proj"], d["b_proj"], dyt)
        r = tm_bwd.tm_linear_bwd(x[t], d["w_proj"], d["b_proj"], dyt, relu=w.tm_kind == wl.TM_LINEAR_RELU)
        return r[0], [], [], r[1], r[2]

    # (1) dense gradient
    dmt.dmt_tower_module_bwd(run.plan, params, run.pooled, run.tm_out, B, dy, dx, arr, ws)
    torch.cuda.synchronize()
    pos = ypos = 0
    for t in range(T):
        dyt = dy[ypos:ypos + B * w.tm_out[t]].reshape(B, -1)
        ref = oracle_bwd(t, to_f64(dyt[sel]))
        got = to_f64(dx[pos:pos + B * tw[t]].reshape(B, -1)[sel])
        assert_grad_close(got, ref[0], rtol, "%s dense grad_pooled tower %d" % (w.name, t))
        assert_grad_close(to_f64(grads[t]["db_proj"]), to_f64(dyt.to(torch.float64).sum(0)), 2e-2,
                          "%s dense db_proj tower %d" % (w.name, t))
        pos += B * tw[t]
        ypos += B * w.tm_out[t]

    # (2) gradient on the sampled samples only
    keep = torch.zeros(B, dtype=torch.bool, device="cuda")
    keep[sel] = True
    ypos = 0
    for t in range(T):
        dy[ypos:ypos + B * w.tm_out[t]].reshape(B, -1)[~keep] = 0.0
        ypos += B * w.tm_out[t]
    dx.fill_(float("nan"))
    # this time on what a training forward kept (cross towers: u_l and x_l; dot towers: the dot terms)
    kept = None
    kept_bytes = dmt.dmt_tm_kept_bytes(run.plan, params, B, w.tm_dtype)
    if kept_bytes:
        kept = torch.empty(kept_bytes, dtype=torch.uint8, device="cuda")
        fws = torch.empty(max(dmt.dmt_tm_workspace_bytes(run.plan, params, B), 256), dtype=torch.uint8, device="cuda")
        y2 = torch.empty_like(run.tm_out)
        dmt.dmt_tower_module_fwd_keep(run.plan, params, run.pooled, B, y2, kept, fws)
        torch.cuda.synchronize()
        assert torch.equal(y2.view(torch.int16), run.tm_out.view(torch.int16))
        del fws, y2
    dmt.dmt_tower_module_bwd(run.plan, params, run.pooled, run.tm_out, B, dy, dx, arr, ws, kept=kept)
    torch.cuda.synchronize()
    pos = ypos = 0
    for t in range(T):
        dyt = dy[ypos:ypos + B * w.tm_out[t]].reshape(B, -1)
        rdx, rdWc, rdbc, rdW, rdb = oracle_bwd(t, to_f64(dyt[sel]))
        dxt = dx[pos:pos + B * tw[t]].reshape(B, -1)
        what = "%s sparse tower %d " % (w.name, t)
        assert_grad_close(to_f64(dxt[sel]), rdx, rtol, what + "grad_pooled")
        assert torch.count_nonzero(dxt[~keep]).item() == 0, what + "other samples' gradients"
        assert_grad_close(to_f64(grads[t]["dw_proj"]), rdW, rtol, what + "dW_proj")
        assert_grad_close(to_f64(grads[t]["db_proj"]), rdb, rtol, what + "db_proj")
        for l in range(nl):
            assert_grad_close(to_f64(grads[t]["dw_cross"][l]), rdWc[l], rtol, what + "dW_cross[%d]" % l)
            assert_grad_close(to_f64(grads[t]["db_cross"][l]), rdbc[l], rtol, what + "db_cross[%d]" % l)
        pos += B * tw[t]
        ypos += B * w.tm_out[t]


def test_interaction_matrix_on_sampled_pairs(run):
    """Tower Partitioner, device stage, on the full batch: entries (i, j) of the interaction
    matrix for sampled feature pairs against the oracle, which pools the two features over all
    B samples itself from the table rows they touch."""
    from oracle import tp
    w, dmt = run.w, run.dmt
    F, B = w.num_tables, w.batch
    if len(set(w.dims)) != 1:
        pytest.skip("tables of different dims have no cosine between them")
    ws = torch.empty(dmt.dmt_tp_workspace_bytes(run.plan, B), dtype=torch.uint8, device="cuda")
    I_dev = torch.empty(F, F, dtype=torch.float32, device="cuda")
    dmt.dmt_tp_interaction(run.plan, run.pooled, B, I_dev, ws)
    torch.cuda.synchronize()
    I = I_dev.cpu().numpy()
    np.testing.assert_array_equal(I, I.T)
    # a feature's cosine with itself is 1 wherever its bag is not empty
    lens = np.diff(run.off).reshape(F, B)
    np.testing.assert_allclose(np.diag(I), (lens > 0).mean(axis=1), atol=1e-4)
    # the table rows as the lookup saw them (the backward run has updated its tables since)
    tables = wl.tables_device(w) if w.backward else run.tables
    rng = np.random.default_rng(321)
    feats = np.sort(rng.choice(F, size=8, replace=False))

    def pooled_of(f):
        seg = run.idx[run.off[f * B]:run.off[(f + 1) * B]]
        rows = np.unique(seg)
        t = tables[f][torch.from_numpy(rows).cuda()]
        vals = t.view(torch.int16).cpu().numpy().view(np.uint16) if w.table_dtype == "bf16" else t.cpu().numpy()
        off = run.off[f * B:(f + 1) * B + 1] - run.off[f * B]
        p = oracle.lookup_towered([vals], w.table_dtype, [w.dims[f]], [0],
                                  np.searchsorted(rows, seg).astype(np.int32), off, B)[0]
        return wl.decode(oracle.round_to(p, w.pooled_dtype), w.pooled_dtype)

    R = np.stack([pooled_of(int(f)) for f in feats], axis=1)            # (B, 8, N)
    ref = tp.tp_interaction(R)
    got = I[np.ix_(feats, feats)]
    # 16-bit pooled values are contracted exactly; what is left is the float32 arithmetic of the
    # cosines and of the batch mean, and the rare pooled element whose float32 sum rounds to the
    # neighbouring 16-bit value
    err = np.abs(got - ref)
    assert err.max() <= 1e-4, (w.name, err.max())
