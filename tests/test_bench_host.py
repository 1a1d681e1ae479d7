"""Host-side pieces of bench.py that need no GPU: the reader of rocprofv3's counter database,
the byte summaries it writes and reads back, and the committed summaries under profiles/."""
import json
import os
import sqlite3
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def _counter_db(path, rows):
    con = sqlite3.connect(path)
    con.execute("create table counters_collection (id integer, kernel_name text, counter_name text, value real)")
    con.executemany("insert into counters_collection values (?, ?, ?, ?)",
                    [(i, k, c, v) for i, (k, c, v) in enumerate(rows)])
    con.commit()
    con.close()


def test_counter_database_is_summed_per_kernel_family(tmp_path):
    db = str(tmp_path / "p_results.db")
    _counter_db(db, [
        ("void (anonymous namespace)::lookup_fwd_kernel<1, 2>(...)", "FETCH_SIZE", 100.0),
        ("void (anonymous namespace)::lookup_fwd_kernel<1, 2>(...)", "FETCH_SIZE", 120.0),
        ("void (anonymous namespace)::bwd_reduce_update_lean<1>(...)", "FETCH_SIZE", 1000.0),
        ("void (anonymous namespace)::radix_scatter(...)", "FETCH_SIZE", 7.0),
        ("dmt_copy_kernel(...)", "FETCH_SIZE", 524288.0),
        ("some_torch_kernel(...)", "FETCH_SIZE", 1e9),          # not a family: ignored
    ])
    got = bench.read_counter_db(db)
    assert got["lookup_fwd"] == [220.0, 2]
    assert got["bwd_reduce_update"] == [1000.0, 1]
    assert got["radix_scatter"] == [7.0, 1]
    assert got["copy"] == [524288.0, 1]
    assert len(got) == 4


def test_traffic_summary_round_trip(tmp_path, monkeypatch):
    scale = {"FETCH_SIZE": 2.0, "WRITE_SIZE": 1.0}
    steps = bench.CHILD_STEPS
    fam = {"copy": {"FETCH_SIZE": (3 * 524288.0, 3), "WRITE_SIZE": (3 * 1048576.0, 3)},
           "lookup_fwd": {"FETCH_SIZE": (steps * 450000.0, steps), "WRITE_SIZE": (steps * 131072.0, steps)}}
    per = {"lookup_fwd": dict(read_bytes=900000 * 1024, write_bytes=131072 * 1024,
                              bytes=(900000 + 131072) * 1024, launches_per_step=1)}
    out = tmp_path / "profiles"
    bench.write_traffic_summary(str(out), "x", ["cmd one", "cmd two"], scale, fam, per, "src")
    text = (out / "bench_x_hbm_traffic.txt").read_text()
    assert "cmd one" in text and "cmd two" in text and "lookup_fwd" in text
    monkeypatch.setattr(bench, "ROOT", str(tmp_path))
    back = bench.committed_traffic("x")
    assert back["per_step"]["lookup_fwd"] == dict(bytes=(900000 + 131072) * 1024, launches_per_step=1)
    assert back["source"].startswith("committed: ")
    assert bench.committed_traffic("no_such_workload") is None


@pytest.mark.parametrize("name", ["backward", "imbalanced", "large"])
def test_committed_byte_summaries_parse(name):
    t = bench.committed_traffic(name)
    assert t is not None, "profiles/bench_%s_hbm_traffic.json is missing" % name
    per = t["per_step"]
    assert "lookup_fwd" in per and per["lookup_fwd"]["bytes"] > 0
    if name != "large":
        assert per["bwd_reduce_update"]["bytes"] > per["bwd_fixup_update"]["bytes"] > 0
    tj = json.load(open(os.path.join(ROOT, "profiles", "bench_%s_hbm_traffic.json" % name)))
    assert abs(tj["fetch_scale"] - 2.0) < 0.05 and abs(tj["write_scale"] - 1.0) < 0.05
