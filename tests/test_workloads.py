"""The synthetic workload generators: shapes, determinism, stated distributions."""
import numpy as np

import workloads as wl


def test_named_configs_have_the_stated_shapes():
    t = wl.tiny()
    assert (t.num_tables, t.num_towers, t.batch, t.dims[0], t.rows[0]) == (8, 2, 64, 16, 1000)
    m = wl.mid()
    assert (m.num_tables, m.num_towers, m.batch) == (64, 8, 8192)
    assert m.tower_widths() == [1024] * 8 and m.tm_in_dims() == [28 + 1024] * 8
    l = wl.large()
    assert l.num_tables == 256 and l.num_towers == 16
    assert [len(x) for x in l.tower_tables()] == [16] * 16
    assert min(l.rows) >= 10_000 and max(l.rows) <= 10_000_000
    cost = [sum(l.rows[f] for f in fs) for fs in l.tower_tables()]
    assert max(cost) / min(cost) < 1.1                      # snake deal balances row x pooling cost
    gb = sum(r * 128 * 2 for r in l.rows) / 1e9
    assert 60 < gb < 130
    i = wl.imbalanced()
    assert [len(x) for x in i.tower_tables()] == wl.IMBALANCED_TOWER_SIZES
    assert set(i.dims) == {32, 64, 128} and i.num_tables == 128
    b = wl.by_name("backward")
    assert b.backward and b.rows == m.rows and b.seed != m.seed


def test_batches_are_seeded_and_well_formed():
    w = wl.scaled(wl.mid(), max_rows=5000, batch=64, num_tables=16)
    a = wl.lookup_batch(w, 0)
    b = wl.lookup_batch(w, 0)
    c = wl.lookup_batch(w, 1)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert not np.array_equal(a[0][:100], c[0][:100])
    idx, off = a
    assert off[0] == 0 and off[-1] == len(idx) and np.all(np.diff(off) >= 0)
    assert np.diff(off).max() <= 100 and abs(np.diff(off).mean() - 20) < 1.0
    for f in range(w.num_tables):
        seg = idx[off[f * w.batch]:off[(f + 1) * w.batch]]
        assert seg.min() >= 0 and seg.max() < w.rows[f]
    # Zipf skew: far fewer distinct ids than lookups
    seg = idx[off[0]:off[w.batch]]
    assert len(np.unique(seg)) < 0.7 * len(seg)


def test_length_distributions():
    t = wl.tiny()
    l = wl.bag_lengths(t)
    assert l.min() == 1 and l.max() == 8
    i = wl.scaled(wl.imbalanced(), max_rows=1000, batch=4096, num_tables=4)
    l = wl.bag_lengths(i)
    assert l.min() == 1 and l.max() <= 500 and 1.8 < l.mean() < 3.5
    assert (l == 1).mean() > 0.55                           # P(floor(X) = 1) = 1 - 2^-1.5 = 0.646


def test_sixteen_bit_round_trip():
    x = np.array([1.0, -2.5, 0.01, 3.14159], dtype=np.float32)
    assert np.array_equal(wl.decode(wl.encode(x, "f32"), "f32"), x.astype(np.float64))
    b = wl.encode(x, "bf16")
    assert b.dtype == np.uint16 and b[0] == 0x3F80
    assert np.allclose(wl.decode(b, "bf16"), x, rtol=2 ** -8)
    assert wl.encode(x, "f16").dtype == np.float16
