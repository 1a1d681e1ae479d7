"""GPU parity of dmt_tower_lookup_fwd against the CPU oracle (through the C ABI)."""
import numpy as np
import pytest
import torch

import oracle
import workloads as wl
from harness import RTOL, DeviceWorkload, assert_close, to_f64

pytestmark = pytest.mark.gpu


def _check(w, out_dtype=None, batch_id=0, env=None):
    dw = DeviceWorkload(w)
    idx, off = wl.lookup_batch(w, batch_id)
    out_dtype = out_dtype or w.pooled_dtype
    got = to_f64(dw.lookup(idx, off, out_dtype))
    assert dw.dmt.dmt_last_device_error(dw.plan) == -1
    ref = oracle.lookup_towered(dw.host_tables, w.table_dtype, w.dims, w.table_to_tower, idx, off, w.batch)
    rtol = RTOL[out_dtype]
    for t, (g, r) in enumerate(zip(dw.split_towers(got), ref)):
        if out_dtype != "f32":
            r = wl.decode(oracle.round_to(r, out_dtype), out_dtype)
        assert_close(g, r, rtol, "%s tower %d" % (w.name, t))


def test_tiny():
    _check(wl.tiny())


@pytest.mark.parametrize("out_dtype", ["bf16", "f16", "f32"])
def test_mid_scaled(out_dtype):
    # 16 tables x 20k rows, two towers, B = 301: several tiles and a ragged tail
    _check(wl.scaled(wl.mid(), max_rows=20000, batch=301, num_tables=16), out_dtype)


def test_large_scaled():
    _check(wl.scaled(wl.large(), max_rows=30000, batch=130, num_tables=40))


def test_imbalanced_scaled():
    _check(wl.scaled(wl.imbalanced(), max_rows=5000, batch=1111, num_tables=24))


@pytest.mark.parametrize("r", [1, 2, 4, 64])
def test_group_shapes_agree(r, monkeypatch):
    """Every rows-in-flight setting of the kernel gives the oracle's result."""
    monkeypatch.setenv("DMT_LOOKUP_R", str(r))
    _check(wl.scaled(wl.mid(), max_rows=3000, batch=77, num_tables=8), "f32")
    _check(wl.scaled(wl.imbalanced(), max_rows=3000, batch=500, num_tables=12), "f32")


@pytest.mark.parametrize("thr", [0, 1, 5, 1000000])
def test_long_bag_threshold_settings_agree(thr, monkeypatch):
    """Bags above the threshold are pooled by a whole wave, the others by their lane group:
    every split (none, all, some, none again) gives the oracle's result."""
    monkeypatch.setenv("DMT_LOOKUP_LONG", str(thr))
    _check(wl.scaled(wl.imbalanced(), max_rows=3000, batch=700, num_tables=12), "f32")
    _check(wl.scaled(wl.mid(), max_rows=3000, batch=77, num_tables=8), "bf16")


def test_empty_bags_and_empty_batch():
    w = wl.scaled(wl.mid(), max_rows=100, batch=9, num_tables=8)
    dw = DeviceWorkload(w)
    off = np.zeros(w.num_tables * w.batch + 1, dtype=np.int64)
    out = dw.lookup(np.zeros(0, dtype=np.int32), off)
    assert torch.count_nonzero(out).item() == 0 and not torch.isnan(out).any()


def test_out_of_range_id_is_reported_not_dereferenced():
    w = wl.scaled(wl.mid(), max_rows=100, batch=16, num_tables=8)
    dw = DeviceWorkload(w)
    idx, off = wl.lookup_batch(w)
    bad = idx.copy()
    bad[37] = 100          # == rows
    bad[91] = -5
    got = to_f64(dw.lookup(bad, off, "f32"))
    assert dw.dmt.dmt_last_device_error(dw.plan) == 37
    assert dw.dmt.dmt_last_device_error(dw.plan) == -1           # cleared
    # the two bad lookups contribute nothing; everything else is intact
    keep = np.ones(len(idx), bool); keep[[37, 91]] = False
    lens = np.diff(off)
    bag_of = np.repeat(np.arange(len(lens)), lens)
    new_off = np.concatenate([[0], np.cumsum(np.bincount(bag_of[keep], minlength=len(lens)))])
    ref = oracle.lookup_towered(dw.host_tables, w.table_dtype, w.dims, w.table_to_tower,
                                idx[keep], new_off, w.batch)
    for g, r in zip(dw.split_towers(got), ref):
        assert_close(g, r, 1e-5, "skip-bad")


@pytest.mark.parametrize("dtype,dim", [("f16", 512), ("f32", 256), ("f16", 8), ("bf16", 24), ("f32", 4)])
def test_row_width_limits(dtype, dim):
    """Rows from one 16-byte chunk (a single lane) to the 1024-byte maximum (a whole wave),
    and a width that is not a power of two."""
    w = wl.scaled(wl.mid(), max_rows=400, batch=37, num_tables=4)
    w.dims = [dim] * 4
    w.table_dtype = dtype
    _check(w, "f32")
    _check(w, dtype)


def test_one_very_long_bag_among_empty_ones():
    w = wl.scaled(wl.mid(), max_rows=1000, batch=5, num_tables=2)
    dw = DeviceWorkload(w, max_nnz=5000)
    rng = np.random.default_rng(3)
    lens = np.zeros(10, dtype=np.int64)
    lens[3] = 3001                                   # table 0, sample 3
    lens[9] = 1                                      # table 1, sample 4
    off = np.concatenate([[0], np.cumsum(lens)])
    idx = rng.integers(0, 1000, size=off[-1]).astype(np.int32)
    got = to_f64(dw.lookup(idx, off, "f32"))
    ref = oracle.lookup_towered(dw.host_tables, w.table_dtype, w.dims, w.table_to_tower, idx, off, w.batch)
    for g, r in zip(dw.split_towers(got), ref):
        assert_close(g, r, 1e-5, "long bag")
