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
