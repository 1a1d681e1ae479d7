"""GPU parity of dmt_tower_module_fwd against the CPU oracle."""
import pytest
import torch

import oracle
import workloads as wl
from harness import RTOL, DeviceWorkload, TowerModules, assert_close, to_device, to_f64

pytestmark = pytest.mark.gpu


def check_tm(w, chained=False):
    """TM on the oracle's pooled values (rounded to the pooled dtype), then
    optionally also the GPU lookup -> GPU TM chain."""
    dw = DeviceWorkload(w)
    tm = TowerModules(dw)
    idx, off = wl.lookup_batch(w)
    pooled = oracle.lookup_towered(dw.host_tables, w.table_dtype, w.dims, w.table_to_tower, idx, off, w.batch)
    enc = [oracle.round_to(p, tm.dtype) for p in pooled]
    x_dev = torch.cat([to_device(e, tm.dtype).reshape(-1) for e in enc])
    got = to_f64(tm.run(x_dev))
    x64 = [wl.decode(e, tm.dtype) for e in enc]
    ref = tm.oracle(x64)
    rtol = RTOL[tm.dtype]
    for t, (g, r) in enumerate(zip(dw.split_towers(got, tm.out_widths), ref)):
        if tm.dtype != "f32":
            r = wl.decode(oracle.round_to(r, tm.dtype), tm.dtype)
        assert_close(g, r, rtol, "%s TM tower %d" % (w.name, t))
    if chained:
        pooled_gpu = dw.lookup(idx, off, tm.dtype)
        got2 = to_f64(tm.run(pooled_gpu))
        for t, (g, r) in enumerate(zip(dw.split_towers(got2, tm.out_widths), ref)):
            if tm.dtype != "f32":
                r = wl.decode(oracle.round_to(r, tm.dtype), tm.dtype)
            assert_close(g, r, rtol if tm.dtype != "f32" else 1e-4, "%s lookup+TM tower %d" % (w.name, t))


def test_tiny_linear_relu_f32():
    check_tm(wl.tiny(), chained=True)


def test_mid_scaled_dot_linear_bf16():
    # 2 towers x 8 features x 128: 28 dots | 1024 -> 256 ; B = 301 leaves ragged M tiles
    check_tm(wl.scaled(wl.mid(), max_rows=5000, batch=301, num_tables=16), chained=True)


def test_large_scaled_cross_linear_bf16():
    # 2 towers of 16 x 128 = 2048 wide: two 2048 x 2048 cross layers, then 2048 -> 512
    w = wl.scaled(wl.large(), max_rows=3000, batch=200)
    sel = [f for f in range(256) if w.table_to_tower[f] in (0, 1)]
    w.rows = [w.rows[f] for f in sel]; w.dims = [128] * 32
    w.table_to_tower = [wl.large().table_to_tower[f] for f in sel]
    w.tm_out = [512, 512]
    check_tm(w, chained=True)


@pytest.mark.parametrize("direct", ["1", "0"])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_cross_linear_on_interior_tiles(direct, dtype, monkeypatch):
    """A batch and widths that are multiples of the 256 x 256 tile: such launches load their
    operand tiles straight into LDS (DMT_TM_DIRECT=0 keeps the register-staged loop); two 1024
    x 1024 cross layers and a 1024 -> 256 projection on two towers, B = 512."""
    monkeypatch.setenv("DMT_TM_DIRECT", direct)
    w = wl.scaled(wl.large(), max_rows=3000, batch=512)
    sel = [f for f in range(256) if w.table_to_tower[f] in (0, 1)][:16]
    w.rows = [w.rows[f] for f in sel]
    w.dims = [128] * 16
    w.table_to_tower = [f // 8 for f in range(16)]
    w.tm_out = [256, 256]
    w.table_dtype = w.pooled_dtype = w.tm_dtype = dtype
    check_tm(w, chained=True)


def test_imbalanced_scaled_linear_f16():
    # towers of unequal width (mixed 32/64/128 dims), Linear -> 128
    check_tm(wl.scaled(wl.imbalanced(), max_rows=2000, batch=777, num_tables=26), chained=True)


def test_dot_linear_odd_feature_count_falls_back():
    # 3 features per tower do not tile a 32-row MFMA block: plain-FMA dot kernel
    w = wl.scaled(wl.mid(), max_rows=500, batch=50, num_tables=6)
    w.table_to_tower = [0, 0, 0, 1, 1, 1]
    w.tm_out = [40, 24]
    check_tm(w)


def test_dot_linear_f32_and_f16():
    w = wl.scaled(wl.mid(), max_rows=500, batch=70, num_tables=8)
    for dt in ("f32", "f16"):
        w.tm_dtype = dt
        w.pooled_dtype = dt
        check_tm(w)


def test_dot_linear_fused_and_separate_towers_in_one_call():
    """Tower 0 (4 features x 64, 6 dots padded to 8, 300 outputs) takes the GEMM that computes
    its dot terms in-kernel; tower 1 (8 features, 96 outputs) the separate dot kernel and the
    128 x 128 GEMM; batch 519 leaves ragged row tiles in both."""
    w = wl.scaled(wl.mid(), max_rows=400, batch=519, num_tables=12)
    w.dims = [64] * 4 + [128] * 8
    w.table_to_tower = [0] * 4 + [1] * 8
    w.tm_out = [300, 96]
    for dt in ("bf16", "f16"):
        w.tm_dtype = dt
        w.pooled_dtype = dt
        check_tm(w)


@pytest.mark.parametrize("out_dim,batch", [(100, 77), (300, 333), (257, 512)])
def test_linear_odd_output_widths_and_ragged_batches(out_dim, batch):
    """Output widths that are no multiple of 8 or of a tile (scalar epilogue, partial
    column tiles) on both GEMM kernels (<= 128 columns: 128 x 128; wider: 256 x 256)."""
    w = wl.scaled(wl.imbalanced(), max_rows=500, batch=batch, num_tables=9)
    w.tm_out = [out_dim] * w.num_towers
    check_tm(w)


def test_cross_with_three_layers_and_narrow_tower():
    w = wl.scaled(wl.large(), max_rows=300, batch=150, num_tables=3)
    w.table_to_tower = [0, 0, 0]
    w.tm_out = [96]
    w.tm_cross_layers = 3
    check_tm(w)                                       # 384-wide cross layers, 96-wide projection


@pytest.mark.parametrize("dt", ["bf16", "f16", "f32"])
def test_dlrm_module_flat_and_shared_per_feature_projection(dt):
    """Listing 1 with c > 0: 2 towers x 8 features x 128, flat 1024 -> 200 next to the shared
    128 -> 24 applied to every feature (200 + 8 * 24 = 392 outputs); batch 301."""
    w = wl.scaled(wl.mid(), max_rows=3000, batch=301, num_tables=16)
    w.tm_kind = wl.TM_DLRM
    w.tm_feat_out = 24
    w.tm_out = [200 + 8 * 24] * 2
    w.tm_dtype = dt
    w.pooled_dtype = dt
    check_tm(w, chained=dt == "bf16")


def test_dlrm_module_odd_widths():
    # 3 features per tower, 20 flat outputs, 5 per feature: nothing is a multiple of 8
    w = wl.scaled(wl.mid(), max_rows=500, batch=77, num_tables=6)
    w.table_to_tower = [0, 0, 0, 1, 1, 1]
    w.tm_kind = wl.TM_DLRM
    w.tm_feat_out = 5
    w.tm_out = [20 + 3 * 5] * 2
    check_tm(w)


@pytest.mark.parametrize("dt,rank", [("bf16", 64), ("bf16", 256), ("f16", 32), ("f32", 5)])
def test_lowrank_cross_module(dt, rank):
    """Two low-rank DCN-v2 cross layers on 512-wide towers (rank 256 takes the 256 x 256 GEMM for
    the second contraction, the smaller ranks the 128 x 128 one), then 512 -> 96; batch 150."""
    w = wl.scaled(wl.large(), max_rows=300, batch=150, num_tables=8)
    w.table_to_tower = [0, 0, 0, 0, 1, 1, 1, 1]
    w.tm_out = [96, 96]
    w.tm_kind = wl.TM_CROSS_LOWRANK_LINEAR
    w.tm_cross_layers = 2
    w.tm_feat_out = rank
    w.tm_dtype = dt
    w.pooled_dtype = dt
    check_tm(w, chained=dt == "bf16" and rank == 64)
