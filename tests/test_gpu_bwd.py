"""GPU parity of dmt_tower_lookup_bwd_update against the CPU oracle."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from harness import RTOL, DeviceWorkload, assert_close, to_f64

pytestmark = pytest.mark.gpu


def run_bwd(dw, idx, off, grad, lr, eps, debug=True):
    dmt, w = dw.dmt, dw.w
    nnz = len(idx)
    d_idx, d_off = torch.from_numpy(idx).cuda(), torch.from_numpy(off).cuda()
    d_grad = torch.from_numpy(grad).cuda()
    ws = torch.empty(max(dmt.dmt_bwd_workspace_bytes(dw.plan, w.batch, nnz), 256) // 8 + 32,
                     dtype=torch.int64, device="cuda")
    ws.fill_(-1)                         # stale scratch must not matter
    dbg = None
    if debug:
        dbg = dict(sorted_keys=torch.full((nnz,), -7, dtype=torch.int64, device="cuda"),
                   sorted_bag=torch.full((nnz,), -7, dtype=torch.int32, device="cuda"),
                   unique_keys=torch.full((nnz,), -7, dtype=torch.int64, device="cuda"),
                   seg_off=torch.full((nnz + 1,), -7, dtype=torch.int64, device="cuda"),
                   num_unique=torch.full((1,), -7, dtype=torch.int64, device="cuda"))
    dmt.dmt_tower_lookup_bwd_update(dw.plan, d_idx, d_off, w.batch, d_grad, lr, eps, ws, debug=dbg)
    torch.cuda.synchronize()
    return dbg


def check_bwd(w, batch_id=0):
    dw = DeviceWorkload(w, with_state=True)
    F, B = w.num_tables, w.batch
    idx, off = wl.lookup_batch(w, batch_id)
    grad = wl.grad_pooled(w, batch_id)
    # non-zero starting state so the accumulate-into-state path is exercised
    rng = np.random.default_rng(99)
    st0 = [rng.random(r).astype(np.float32) * 1e-3 for r in w.rows]
    for s, h in zip(dw.states, st0):
        s.copy_(torch.from_numpy(h))
    before = [t.clone() for t in dw.tables]
    dbg = run_bwd(dw, idx, off, grad, w.lr, w.eps)
    assert dw.dmt.dmt_last_device_error(dw.plan) == -1

    # integer stages: bit exact
    st, sr, sp = oracle.sort_keys(F, B, idx, off)
    bag_of_pos = np.repeat(np.arange(F * B), np.diff(off))
    ut, ur, so = oracle.unique(st, sr)
    U = int(dbg["num_unique"].item())
    assert U == len(ut)
    assert np.array_equal(dbg["sorted_keys"].cpu().numpy(), (st << 32) | sr)
    assert np.array_equal(dbg["sorted_bag"].cpu().numpy(), bag_of_pos[sp].astype(np.int32))
    assert np.array_equal(dbg["unique_keys"].cpu().numpy()[:U], (ut << 32) | ur)
    assert np.array_equal(dbg["seg_off"].cpu().numpy()[:U + 1], so)

    # floating-point stages
    ref = oracle.bwd_update(dw.host_tables, w.table_dtype, st0, w.dims, w.table_to_tower, idx, off,
                            B, grad, w.lr, w.eps)
    assert np.array_equal(ref["key_table"], ut) and np.array_equal(ref["key_row"], ur)
    rtol = RTOL[w.table_dtype]
    for f in range(F):
        m = ref["key_table"] == f
        rows = ref["key_row"][m]
        D = w.dims[f]
        got_rows = to_f64(dw.tables[f][torch.from_numpy(rows).cuda()])
        want = ref["new_rows"][m][:, :D]
        if w.table_dtype != "f32":
            want = wl.decode(oracle.round_to(want, w.table_dtype), w.table_dtype)
        assert_close(got_rows, want, rtol, "%s rows of table %d" % (w.name, f))
        got_state = to_f64(dw.states[f][torch.from_numpy(rows).cuda()])
        assert_close(got_state, ref["new_state"][m].astype(np.float32), 1e-5, "state of table %d" % f)
        # rows no lookup touched are bit-identical, and so are their states
        untouched = np.ones(w.rows[f], bool)
        untouched[rows] = False
        ut_idx = torch.from_numpy(np.nonzero(untouched)[0]).cuda()
        assert torch.equal(dw.tables[f][ut_idx].view(torch.int16 if D and w.table_dtype != "f32" else torch.int32),
                           before[f][ut_idx].view(torch.int16 if w.table_dtype != "f32" else torch.int32))
        assert torch.equal(dw.states[f][ut_idx].cpu(), torch.from_numpy(st0[f])[ut_idx.cpu()])
    return dw, idx, off, grad, st0, before


def test_tiny():
    check_bwd(wl.tiny())


def test_mid_scaled_and_repeatable():
    w = wl.scaled(wl.mid(True), max_rows=20000, batch=301, num_tables=16)
    dw, idx, off, grad, st0, before = check_bwd(w)
    first_t = [t.clone() for t in dw.tables]
    first_s = [s.clone() for s in dw.states]
    # same inputs again from the same starting point: same bits
    for t, b in zip(dw.tables, before):
        t.copy_(b)
    for s, h in zip(dw.states, st0):
        s.copy_(torch.from_numpy(h))
    run_bwd(dw, idx, off, grad, w.lr, w.eps, debug=False)
    for a, b in zip(dw.tables, first_t):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
    for a, b in zip(dw.states, first_s):
        assert torch.equal(a, b)


@pytest.mark.parametrize("kernel", ["1", "2"])
def test_the_other_segment_reduce_kernels(kernel, monkeypatch):
    # rows of at most 128 columns take the lean walk; the wave-per-tile and lane-group walks
    # (wider rows) are reached here through the plan's switch
    monkeypatch.setenv("DMT_BWD_KERNEL", kernel)
    check_bwd(wl.scaled(wl.mid(True), max_rows=3000, batch=300, num_tables=12))
    check_bwd(wl.scaled(wl.imbalanced(), max_rows=2000, batch=400, num_tables=20))


def test_hot_rows_span_many_tiles():
    # 200 rows only: every row is hit thousands of times, runs cross many reduce tiles
    check_bwd(wl.scaled(wl.mid(True), max_rows=200, batch=512, num_tables=8))


def test_imbalanced_scaled_mixed_dims():
    check_bwd(wl.scaled(wl.imbalanced(), max_rows=5000, batch=1111, num_tables=24))


@pytest.mark.parametrize("dims", [[32, 64], [64], [32], [256]])
def test_narrow_and_wide_rows(dims):
    """Dims up to 128 run the lean walk, 256 the wave-per-tile kernel."""
    w = wl.scaled(wl.imbalanced(), max_rows=3000, batch=400, num_tables=12)
    w.dims = [dims[f % len(dims)] for f in range(12)]
    check_bwd(w)


@pytest.mark.parametrize("widest", [136, 160, 200, 248])
def test_widest_row_between_128_and_256_columns(widest):
    """Mixed widths whose widest row is neither 128 nor 256 columns take the lane-group walk with
    64-lane groups of which only widest / 4 lanes hold columns; the records of the other lanes
    count like any other (they once did not: their gradients were dropped)."""
    w = wl.scaled(wl.imbalanced(), max_rows=700, batch=150, num_tables=9)
    w.dims = [widest, 64, 16, 128, widest, 32, 8, 96, 24]
    check_bwd(w)


def test_large_scaled_bf16():
    w = wl.scaled(wl.large(), max_rows=30000, batch=130, num_tables=40)
    w.backward = True
    check_bwd(w)


def test_many_small_tables_some_without_lookups():
    """300 tables (more than one pass of the sort-block map's 256-table chunks), a few rows each,
    Poisson(0.3) bag lengths so that many tables have no lookup at all in a batch of 3."""
    base = wl.scaled(wl.imbalanced(), max_rows=60, batch=3, num_tables=100)
    w = wl.dataclasses.replace(
        base, rows=[7 + (f * 13) % 50 for f in range(300)], dims=[32] * 300,
        table_to_tower=[f // 25 for f in range(300)], tm_out=[128] * 12, len_dist="poisson",
        len_param=0.3, len_cap=3, zipf_alpha=None)
    check_bwd(w)


def test_empty_batch_is_a_no_op():
    w = wl.scaled(wl.mid(True), max_rows=100, batch=9, num_tables=8)
    dw = DeviceWorkload(w, with_state=True)
    before = [t.clone() for t in dw.tables]
    off = np.zeros(w.num_tables * w.batch + 1, dtype=np.int64)
    dbg = run_bwd(dw, np.zeros(0, np.int32), off, wl.grad_pooled(w), 0.01, 1e-8)
    assert int(dbg["num_unique"].item()) == 0 and int(dbg["seg_off"][0].item()) == 0
    for a, b in zip(dw.tables, before):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))


def test_out_of_range_ids_are_skipped():
    w = wl.scaled(wl.mid(True), max_rows=100, batch=16, num_tables=8)
    dw = DeviceWorkload(w, with_state=True)
    idx, off = wl.lookup_batch(w)
    grad = wl.grad_pooled(w)
    bad = idx.copy()
    bad[[5, 700]] = [100, -1]
    dbg = run_bwd(dw, bad, off, grad, w.lr, w.eps)
    assert dw.dmt.dmt_last_device_error(dw.plan) == 5
    keep = np.ones(len(idx), bool); keep[[5, 700]] = False
    lens = np.diff(off)
    bag_of = np.repeat(np.arange(len(lens)), lens)
    new_off = np.concatenate([[0], np.cumsum(np.bincount(bag_of[keep], minlength=len(lens)))])
    st0 = [np.zeros(r, np.float32) for r in w.rows]
    ref = oracle.bwd_update(dw.host_tables, w.table_dtype, st0, w.dims, w.table_to_tower,
                            idx[keep], new_off, w.batch, grad, w.lr, w.eps)
    assert int(dbg["num_unique"].item()) == len(ref["key_row"])
    for f in range(w.num_tables):
        m = ref["key_table"] == f
        rows = ref["key_row"][m]
        want = wl.decode(oracle.round_to(ref["new_rows"][m][:, :w.dims[f]], "f16"), "f16")
        assert_close(to_f64(dw.tables[f][torch.from_numpy(rows).cuda()]), want, 2e-2, "rows")


@pytest.mark.parametrize("case", ["first_not_zero", "descending", "last_not_nnz", "beyond_nnz"])
def test_malformed_offsets_update_nothing_and_are_reported(case):
    # the host cannot see device offsets; the key build checks them and the update is skipped
    w = wl.scaled(wl.mid(True), max_rows=100, batch=16, num_tables=8)
    dw = DeviceWorkload(w, with_state=True)
    idx, off = wl.lookup_batch(w)
    grad = wl.grad_pooled(w)
    bad = off.copy()
    nbags = len(off) - 1
    if case == "first_not_zero":
        bad[0], where = 3, 0
    elif case == "descending":
        bad[41], where = bad[40] - 1 if bad[40] > 0 else bad[42] + 1, 40
        if bad[41] > bad[42]:
            where = 41
    elif case == "last_not_nnz":
        bad[-1], where = len(idx) - 2, nbags - 1
    else:
        bad[-1], where = len(idx) + 5, nbags - 1
    before = [t.clone() for t in dw.tables]
    run_bwd(dw, idx, bad, grad, w.lr, w.eps, debug=False)
    with pytest.raises(dw.dmt.DmtError) as e:
        dw.dmt.dmt_last_device_error(dw.plan)
    assert e.value.code == 1 and e.value.position == where           # DMT_EINVAL, first bad bag
    for a, b, s in zip(dw.tables, before, dw.states):
        assert torch.equal(a.view(torch.int16), b.view(torch.int16))
        assert int((s != 0).sum()) == 0
    # the record is cleared and a well-formed call works afterwards
    run_bwd(dw, idx, off, grad, w.lr, w.eps, debug=False)
    assert dw.dmt.dmt_last_device_error(dw.plan) == -1
    assert sum(int((s != 0).sum()) for s in dw.states) > 0


def _degenerate(ids_of):
    w = wl.scaled(wl.mid(True), max_rows=5000, batch=64, num_tables=2)
    w.table_to_tower = [0, 0]
    w.tm_out = [256]
    dw = DeviceWorkload(w, with_state=True)
    lens = np.full(2 * 64, 30, dtype=np.int64)
    off = np.concatenate([[0], np.cumsum(lens)])
    idx = ids_of(int(off[-1])).astype(np.int32)
    grad = wl.grad_pooled(w)
    dbg = run_bwd(dw, idx, off, grad, w.lr, w.eps)
    st0 = [np.zeros(r, np.float32) for r in w.rows]
    ref = oracle.bwd_update(dw.host_tables, w.table_dtype, st0, w.dims, w.table_to_tower, idx, off,
                            w.batch, grad, w.lr, w.eps)
    assert int(dbg["num_unique"].item()) == len(ref["key_row"])
    for f in range(2):
        m = ref["key_table"] == f
        rows = torch.from_numpy(ref["key_row"][m]).cuda()
        want = wl.decode(oracle.round_to(ref["new_rows"][m][:, :128], "f16"), "f16")
        assert_close(to_f64(dw.tables[f][rows]), want, 2e-2, "rows")
        assert_close(to_f64(dw.states[f][rows]), ref["new_state"][m], 1e-5, "state")


def test_every_lookup_hits_the_same_row():
    # one run per table as long as the table's whole record range: 15 reduce tiles chained
    _degenerate(lambda n: np.full(n, 17))


def test_every_lookup_hits_a_different_row():
    # no duplicates at all: every run has length one
    _degenerate(lambda n: np.arange(n) % 1920 + (np.arange(n) // 1920) * 0)
