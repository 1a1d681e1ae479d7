"""Seeded random configurations (table counts, widths, row counts, batch sizes, bag-length and
id distributions, dtypes, tower assignments) through the lookup and the update, each against
the oracle: shapes nobody thought of when writing the other tests."""
import dataclasses

import numpy as np
import pytest

import workloads as wl
from test_gpu_bwd import check_bwd
from test_gpu_lookup import _check as check_lookup

pytestmark = pytest.mark.gpu

DIMS = {"f16": [8, 16, 24, 32, 48, 64, 96, 128, 160, 256], "bf16": [8, 16, 32, 64, 72, 128, 200, 256],
        "f32": [4, 8, 12, 16, 32, 64, 100, 128, 256]}


def random_workload(seed):
    rng = np.random.default_rng([77, seed])
    dt = ["f16", "bf16", "f32"][int(rng.integers(3))]
    F = int(rng.integers(1, 15))
    T = int(rng.integers(1, min(F, 4) + 1))
    # every tower gets at least one table, the rest at random
    t2t = list(range(T)) + [int(x) for x in rng.integers(0, T, size=F - T)]
    t2t = [int(x) for x in rng.permutation(t2t)]
    same_dim = rng.random() < 0.4
    dims = [int(rng.choice(DIMS[dt]))] * F if same_dim else [int(rng.choice(DIMS[dt])) for _ in range(F)]
    rows = [int(np.exp(rng.uniform(0, np.log(4000)))) for _ in range(F)]
    dist = ["uniform", "poisson", "pareto"][int(rng.integers(3))]
    param = {"uniform": float(rng.integers(1, 9)), "poisson": float(rng.choice([0.3, 2.0, 9.0, 30.0])),
             "pareto": 1.5}[dist]
    base = wl.scaled(wl.imbalanced(), max_rows=10, batch=4, num_tables=1)
    return dataclasses.replace(
        base, name="random%d" % seed, seed=1000 + seed, rows=rows, dims=dims, table_dtype=dt,
        table_to_tower=t2t, batch=int(np.exp(rng.uniform(0, np.log(700)))), len_dist=dist,
        len_param=param, len_cap=max(int(rng.choice([3, 40, 400])), int(param)),
        zipf_alpha=None if rng.random() < 0.5 else 1.05, tm_out=[128] * T,
        pooled_dtype=dt if rng.random() < 0.5 else "f32", tm_dtype=dt, backward=True)


@pytest.mark.parametrize("seed", range(64))
def test_random_configuration(seed):
    w = random_workload(seed)
    check_lookup(w)
    check_bwd(w)


@pytest.mark.parametrize("seed", range(16))
def test_random_configuration_with_ids_outside_their_tables(seed):
    """About one lookup in fifty names a row its table does not have (negative, or past the
    end): the lookup and the update must behave exactly as if those lookups were not there,
    and report the first of them."""
    import torch
    import oracle
    from harness import RTOL, DeviceWorkload, assert_close, to_f64
    from test_gpu_bwd import run_bwd

    w = random_workload(500 + seed)
    rng = np.random.default_rng([78, seed])
    idx, off = wl.lookup_batch(w, 0)
    if len(idx) == 0:
        pytest.skip("no lookups drawn")
    F, B = w.num_tables, w.batch
    lens = np.diff(off)
    bag_of = np.repeat(np.arange(F * B), lens)
    nbad = max(1, len(idx) // 50)
    bad_pos = np.sort(rng.choice(len(idx), size=nbad, replace=False))
    bad = idx.copy()
    rows_of = np.asarray(w.rows)[bag_of[bad_pos] // B]
    kind = rng.integers(0, 4, nbad)                  # just past the end, just below zero, the extremes
    bad[bad_pos] = np.select([kind == 0, kind == 1, kind == 2],
                             [rows_of + rng.integers(0, 5, nbad), -1 - rng.integers(0, 5, nbad),
                              np.full(nbad, 2**31 - 1)], np.full(nbad, -2**31)).astype(np.int32)
    keep = np.ones(len(idx), bool)
    keep[bad_pos] = False
    clean_idx = np.ascontiguousarray(idx[keep])
    clean_off = np.concatenate([[0], np.cumsum(np.bincount(bag_of[keep], minlength=F * B))]).astype(np.int64)

    dw = DeviceWorkload(w, with_state=True)
    got = to_f64(dw.lookup(bad, off, "f32"))
    assert dw.dmt.dmt_last_device_error(dw.plan) == int(bad_pos[0])
    ref = oracle.lookup_towered(dw.host_tables, w.table_dtype, w.dims, w.table_to_tower, clean_idx,
                                clean_off, B)
    for t, (g, r) in enumerate(zip(dw.split_towers(got), ref)):
        assert_close(g, r, 1e-5, "lookup tower %d" % t)

    grad = wl.grad_pooled(w, 0)
    before = [t.clone() for t in dw.tables]
    run_bwd(dw, bad, off, grad, w.lr, w.eps, debug=False)
    assert dw.dmt.dmt_last_device_error(dw.plan) == int(bad_pos[0])
    st0 = [np.zeros(r, np.float32) for r in w.rows]
    want = oracle.bwd_update(dw.host_tables, w.table_dtype, st0, w.dims, w.table_to_tower, clean_idx,
                             clean_off, B, grad, w.lr, w.eps)
    for f in range(F):
        m = want["key_table"] == f
        rows = want["key_row"][m]
        D = w.dims[f]
        new_rows = want["new_rows"][m][:, :D]
        if w.table_dtype != "f32":
            new_rows = wl.decode(oracle.round_to(new_rows, w.table_dtype), w.table_dtype)
        sel = torch.from_numpy(rows).cuda()
        assert_close(to_f64(dw.tables[f][sel]), new_rows, RTOL[w.table_dtype], "rows of table %d" % f)
        assert_close(to_f64(dw.states[f][sel]), want["new_state"][m].astype(np.float32), 1e-5,
                     "state of table %d" % f)
        untouched = np.ones(w.rows[f], bool)
        untouched[rows] = False
        u = torch.from_numpy(np.nonzero(untouched)[0]).cuda()
        bits = torch.int16 if w.table_dtype != "f32" else torch.int32
        assert torch.equal(dw.tables[f][u].view(bits), before[f][u].view(bits))
        assert torch.count_nonzero(dw.states[f][u]).item() == 0


@pytest.mark.parametrize("kernel", ["1", "2"])
@pytest.mark.parametrize("seed", range(100, 120))
def test_random_configuration_on_the_other_segment_reduce_kernels(seed, kernel, monkeypatch):
    """The same arbitrary configurations with the plan's switch set to the wave-per-tile walk
    (taken where the widest row has 128 or 256 columns) and to the lane-group walk."""
    monkeypatch.setenv("DMT_BWD_KERNEL", kernel)
    check_bwd(random_workload(seed))


@pytest.mark.parametrize("seed", range(8))
def test_random_configuration_with_many_rows(seed):
    """Tables of up to 400 000 rows: ids need 17 to 19 bits, so the sort takes three passes, and
    most lookups hit rows of their own."""
    rng = np.random.default_rng([79, seed])
    w = random_workload(300 + seed)
    F = min(w.num_tables, 5)
    w = dataclasses.replace(
        w, rows=[int(np.exp(rng.uniform(np.log(70000), np.log(400000)))) for _ in range(F)],
        dims=[min(d, 64) for d in w.dims[:F]], table_to_tower=[0] * F, tm_out=[128],
        batch=int(rng.integers(200, 900)))
    check_lookup(w)
    check_bwd(w)


@pytest.mark.parametrize("seed", range(24))
def test_random_configuration_with_random_lookup_switches(seed, monkeypatch):
    """The lookup's launch shape (row slots per bag, bags a lane group pools in turn, the
    threshold from which a bag goes to a whole wave) set at random instead of derived."""
    rng = np.random.default_rng([80, seed])
    monkeypatch.setenv("DMT_LOOKUP_R", str(int(rng.choice([0, 1, 2, 4, 8]))))
    monkeypatch.setenv("DMT_LOOKUP_BPG", str(int(rng.choice([0, 1, 2, 3, 8, 16, 64]))))
    monkeypatch.setenv("DMT_LOOKUP_LONG", str(int(rng.choice([-1, 0, 1, 5, 60]))))
    check_lookup(random_workload(700 + seed))


@pytest.mark.parametrize("seed", range(12))
def test_random_configuration_with_few_rows_and_many_lookups(seed):
    """Tables of 1 to 60 rows under batches of up to 3000 samples: every row's run spans many
    reduce tiles, so most of the work goes through the partial sums and the fix-up."""
    rng = np.random.default_rng([81, seed])
    w = random_workload(1200 + seed)
    w = dataclasses.replace(w, rows=[int(np.exp(rng.uniform(0, np.log(60)))) for _ in w.rows],
                            batch=int(rng.integers(500, 3000)), len_cap=max(w.len_cap, 40))
    check_bwd(w)
