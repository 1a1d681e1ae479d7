"""GPU parity of dmt_tower_module_bwd against the CPU oracle (oracle/tm_bwd.py).

Both sides start from the same encoded values: the pooled block and the weights rounded to the
compute dtype, and a float32 N(0,1) gradient of the module outputs.  The oracle differentiates
in float64; the library rounds its contraction operands once to the compute dtype, which the
tolerance (relative to each output's magnitude plus the array's rms) covers.
"""
import numpy as np
import pytest
import torch

import oracle
from oracle import tm_bwd
import workloads as wl
from harness import (RTOL, DeviceWorkload, TowerModules, assert_close, assert_grad_close, to_device,
                     to_f64)

pytestmark = pytest.mark.gpu


def run_bwd(dw, tm, x_dev, y_dev, dy_dev, kept=None):
    """Calls the library; returns (grad_pooled flat float64, per-tower dicts of float64 grads)."""
    w = dw.w
    dmt = dw.dmt
    nan = float("nan")
    widths = w.tower_widths()
    grads = []
    for t, kin in enumerate(w.tm_in_dims()):
        L = w.tm_cross_layers if w.tm_kind == wl.TM_CROSS_LINEAR else 0
        f = lambda *shape: torch.full(shape, nan, dtype=torch.float32, device="cuda")
        if w.tm_kind == wl.TM_DLRM:
            nf = len(w.tower_tables()[t])
            o_proj = w.tm_out[t] - nf * w.tm_feat_out
            grads.append(dict(dw_proj=f(o_proj, kin), db_proj=f(o_proj),
                              dw_cross=[f(w.tm_feat_out, widths[t] // nf)], db_cross=[f(w.tm_feat_out)]))
            continue
        if w.tm_kind == wl.TM_CROSS_LOWRANK_LINEAR:
            r, d = w.tm_feat_out, widths[t]
            grads.append(dict(dw_proj=f(w.tm_out[t], kin), db_proj=f(w.tm_out[t]),
                              dw_cross=[f(*shape) for _ in range(w.tm_cross_layers) for shape in ((r, d), (d, r))],
                              db_cross=[f(d) for _ in range(w.tm_cross_layers)]))
            continue
        grads.append(dict(dw_proj=f(w.tm_out[t], kin), db_proj=f(w.tm_out[t]),
                          dw_cross=[f(widths[t], widths[t]) for _ in range(L)],
                          db_cross=[f(widths[t]) for _ in range(L)]))
    arr = dmt.make_tm_grads(grads)
    nbytes = dmt.dmt_tm_bwd_workspace_bytes(dw.plan, tm.params, w.batch)
    assert nbytes > 0
    ws = torch.empty(nbytes // 8 + 32, dtype=torch.int64, device="cuda")
    dx = torch.full((w.batch * sum(widths),), nan, dtype=torch.float32, device="cuda")
    dmt.dmt_tower_module_bwd(dw.plan, tm.params, x_dev, y_dev, w.batch, dy_dev, dx, arr, ws, kept=kept)
    torch.cuda.synchronize()
    host = [dict(dw_proj=to_f64(g["dw_proj"]), db_proj=to_f64(g["db_proj"]),
                 dw_cross=[to_f64(a) for a in g["dw_cross"]],
                 db_cross=[to_f64(a) for a in g["db_cross"]]) for g in grads]
    return to_f64(dx), host


def forward_keep(dw, tm, x_dev):
    """dmt_tower_module_fwd_keep; checks its output against the plain forward's, bit for bit."""
    w, dmt = dw.w, dw.dmt
    nbytes = dmt.dmt_tm_kept_bytes(dw.plan, tm.params, w.batch, tm.dtype)
    kept = torch.full((nbytes // 2 + 128,), -1, dtype=torch.int16, device="cuda") if nbytes else None
    y = torch.full((w.batch * sum(tm.out_widths),), float("nan"), dtype=x_dev.dtype, device="cuda")
    dmt.dmt_tower_module_fwd_keep(dw.plan, tm.params, x_dev, w.batch, y, kept, tm.workspace)
    torch.cuda.synchronize()
    plain = tm.run(x_dev)
    bits = torch.int32 if y.dtype == torch.float32 else torch.int16
    assert torch.equal(y.view(bits), plain.view(bits))
    return kept


def check_tm_bwd(w, rtol=None, keep=False):
    dw = DeviceWorkload(w)
    tm = TowerModules(dw)
    idx, off = wl.lookup_batch(w)
    pooled = oracle.lookup_towered(dw.host_tables, w.table_dtype, w.dims, w.table_to_tower, idx, off, w.batch)
    enc = [oracle.round_to(p, tm.dtype) for p in pooled]
    x_dev = torch.cat([to_device(e, tm.dtype).reshape(-1) for e in enc])
    x64 = [wl.decode(e, tm.dtype) for e in enc]
    dy_all = wl.grad_tm_out(w)
    dys, o = [], 0
    for t in range(w.num_towers):
        dys.append(dy_all[o:o + w.batch * w.tm_out[t]].reshape(w.batch, w.tm_out[t]).copy())
        o += w.batch * w.tm_out[t]
    if w.tm_kind == wl.TM_LINEAR_RELU:
        # an output whose pre-activation is a rounding error away from zero may be on in one
        # arithmetic and off in the other: such outputs receive no gradient in this test
        for t in range(w.num_towers):
            pre = oracle.tm_linear(x64[t], tm.dec[t]["w_proj"], tm.dec[t]["b_proj"])
            dys[t][np.abs(pre) < 1e-3 * np.sqrt(np.mean(pre * pre))] = 0.0
    dy_dev = torch.from_numpy(np.concatenate([d.reshape(-1) for d in dys])).cuda()
    y_dev = tm.run(x_dev) if w.tm_kind == wl.TM_LINEAR_RELU else None
    kept = forward_keep(dw, tm, x_dev) if keep else None
    got_dx, got = run_bwd(dw, tm, x_dev, y_dev, dy_dev, kept)
    rtol = rtol or RTOL[tm.dtype]
    tables = w.tower_tables()
    for t, gdx in enumerate(dw.split_towers(got_dx, w.tower_widths())):
        d = tm.dec[t]
        what = "%s TM backward tower %d " % (w.name, t)
        if w.tm_kind in (wl.TM_LINEAR, wl.TM_LINEAR_RELU):
            dx, dW, db = tm_bwd.tm_linear_bwd(x64[t], d["w_proj"], d["b_proj"], dys[t],
                                              relu=w.tm_kind == wl.TM_LINEAR_RELU)
        elif w.tm_kind == wl.TM_DOT_LINEAR:
            dx, dW, db = tm_bwd.tm_dot_linear_bwd(x64[t], len(tables[t]), d["w_proj"], d["b_proj"], dys[t])
        elif w.tm_kind == wl.TM_CROSS_LOWRANK_LINEAR:
            dx, dVc, dUc, dbc, dW, db = tm_bwd.tm_cross_lowrank_linear_bwd(
                x64[t], d["w_cross"][0::2], d["w_cross"][1::2], d["b_cross"], d["w_proj"], d["b_proj"], dys[t])
            for l in range(len(dVc)):
                assert_grad_close(got[t]["dw_cross"][2 * l], dVc[l], rtol, what + "dV[%d]" % l)
                assert_grad_close(got[t]["dw_cross"][2 * l + 1], dUc[l], rtol, what + "dU[%d]" % l)
                assert_grad_close(got[t]["db_cross"][l], dbc[l], rtol, what + "db_cross[%d]" % l)
        elif w.tm_kind == wl.TM_DLRM:
            dx, dW, db, dWf, dbf = tm_bwd.tm_dlrm_bwd(x64[t], len(tables[t]), d["w_proj"], d["b_proj"],
                                                      d["w_cross"][0], d["b_cross"][0], dys[t])
            assert_grad_close(got[t]["dw_cross"][0], dWf, rtol, what + "dW_feat")
            pD = d["w_proj"].shape[0]
            assert_grad_close(got[t]["db_cross"][0], dbf, rtol, what + "db_feat",
                              scale=np.abs(dys[t][:, pD:]).reshape(w.batch, len(tables[t]), -1).sum((0, 1)))
        else:
            dx, dWc, dbc, dW, db = tm_bwd.tm_cross_linear_bwd(x64[t], d["w_cross"], d["b_cross"],
                                                              d["w_proj"], d["b_proj"], dys[t])
            for l in range(len(dWc)):
                assert_grad_close(got[t]["dw_cross"][l], dWc[l], rtol, what + "dW_cross[%d]" % l)
                assert_grad_close(got[t]["db_cross"][l], dbc[l], rtol, what + "db_cross[%d]" % l)
        assert_grad_close(gdx, dx, rtol, what + "grad_pooled")
        assert_grad_close(got[t]["dw_proj"], dW, rtol, what + "dW_proj")
        assert_grad_close(got[t]["db_proj"], db, rtol, what + "db_proj",
                          scale=np.abs(dys[t][:, :len(db)]).sum(0))


def test_tiny_linear_relu_f32():
    check_tm_bwd(wl.tiny())


def test_linear_bf16_and_f16_ragged():
    # towers of unequal width, batch 777 (not a multiple of 8: padded transposed operands),
    # output width 100 (padded gradient operand, partial column tiles)
    w = wl.scaled(wl.imbalanced(), max_rows=2000, batch=777, num_tables=26)
    w.tm_out = [100] * w.num_towers
    for dt in ("f16", "bf16"):
        w.tm_dtype = dt
        w.pooled_dtype = dt
        check_tm_bwd(w)


def test_linear_relu_bf16_wide_output():
    w = wl.scaled(wl.imbalanced(), max_rows=500, batch=333, num_tables=9)
    w.tm_kind = wl.TM_LINEAR_RELU
    w.tm_out = [300] * w.num_towers
    check_tm_bwd(w)


def test_mid_scaled_dot_linear_bf16():
    # 2 towers x 8 features x 128: 28 dots (padded to 32) | 1024 -> 256; batch 301
    check_tm_bwd(wl.scaled(wl.mid(), max_rows=5000, batch=301, num_tables=16))


def test_dot_linear_odd_feature_count_f32_and_f16():
    w = wl.scaled(wl.mid(), max_rows=500, batch=50, num_tables=6)
    w.table_to_tower = [0, 0, 0, 1, 1, 1]
    w.tm_out = [40, 24]
    for dt in ("f32", "f16"):
        w.tm_dtype = dt
        w.pooled_dtype = dt
        check_tm_bwd(w)


def test_large_scaled_cross_linear_bf16():
    # 2 towers of 16 x 128 = 2048 wide: two 2048 x 2048 cross layers, then 2048 -> 512
    w = wl.scaled(wl.large(), max_rows=3000, batch=200)
    sel = [f for f in range(256) if w.table_to_tower[f] in (0, 1)]
    w.rows = [w.rows[f] for f in sel]; w.dims = [128] * 32
    w.table_to_tower = [wl.large().table_to_tower[f] for f in sel]
    w.tm_out = [512, 512]
    check_tm_bwd(w, rtol=4e-2)


@pytest.mark.parametrize("keep", [False, True])
def test_cross_three_layers_narrow_tower_f32_and_bf16(keep):
    """keep: the cross layers' u_l and x_l come from dmt_tower_module_fwd_keep instead of being
    recomputed by the backward."""
    w = wl.scaled(wl.large(), max_rows=300, batch=150, num_tables=3)
    w.table_to_tower = [0, 0, 0]
    w.tm_out = [96]
    w.tm_cross_layers = 3
    for dt, rtol in (("f32", 1e-4), ("bf16", 4e-2)):
        w.tm_dtype = dt
        w.pooled_dtype = dt
        check_tm_bwd(w, rtol, keep=keep)


def test_kept_activations_wide_cross_tower_and_dot_towers():
    # two 2048-wide towers (256 x 256 GEMM path), 2 layers; then dot towers, whose training forward
    # keeps the dot terms it computes inside the projection kernel
    w = wl.scaled(wl.large(), max_rows=3000, batch=200)
    sel = [f for f in range(256) if w.table_to_tower[f] in (0, 1)]
    w.rows = [w.rows[f] for f in sel]; w.dims = [128] * 32
    w.table_to_tower = [wl.large().table_to_tower[f] for f in sel]
    w.tm_out = [512, 512]
    check_tm_bwd(w, rtol=4e-2, keep=True)
    check_tm_bwd(wl.scaled(wl.mid(), max_rows=5000, batch=301, num_tables=16), keep=True)


@pytest.mark.parametrize("dt,fuse", [("f32", "1"), ("f16", "1"), ("bf16", "0")])
def test_kept_dot_terms_on_every_dot_path(dt, fuse, monkeypatch):
    """The dot terms a training forward keeps, from the one-thread-per-term kernel (float32), the
    fused projection kernel, and the separate Gram-tile kernel (fusion switched off); 5 features
    per tower leave padding columns behind the 10 terms."""
    monkeypatch.setenv("DMT_TM_FUSE", fuse)
    w = wl.scaled(wl.mid(), max_rows=3000, batch=257, num_tables=16)
    w.tm_dtype = dt
    w.pooled_dtype = dt
    check_tm_bwd(w, rtol=1e-4 if dt == "f32" else 4e-2, keep=True)
    w5 = wl.scaled(wl.mid(), max_rows=3000, batch=130, num_tables=10)
    w5.table_to_tower = [0] * 5 + [1] * 5
    w5.tm_out = [256, 256]
    w5.tm_dtype = dt
    w5.pooled_dtype = dt
    check_tm_bwd(w5, rtol=1e-4 if dt == "f32" else 4e-2, keep=True)


@pytest.mark.parametrize("dt", ["bf16", "f16", "f32"])
def test_dlrm_module_flat_and_shared_per_feature_projection(dt):
    # 2 towers x 8 features x 128: flat 1024 -> 200 next to the shared 128 -> 24 (392 outputs)
    w = wl.scaled(wl.mid(), max_rows=3000, batch=301, num_tables=16)
    w.tm_kind = wl.TM_DLRM
    w.tm_feat_out = 24
    w.tm_out = [200 + 8 * 24] * 2
    w.tm_dtype = dt
    w.pooled_dtype = dt
    check_tm_bwd(w)


def test_dlrm_module_odd_widths():
    w = wl.scaled(wl.mid(), max_rows=500, batch=77, num_tables=6)
    w.table_to_tower = [0, 0, 0, 1, 1, 1]
    w.tm_kind = wl.TM_DLRM
    w.tm_feat_out = 5
    w.tm_out = [20 + 3 * 5] * 2
    check_tm_bwd(w)


@pytest.mark.parametrize("kind", ["linear_relu", "dot_linear", "cross_linear", "dlrm"])
@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_degenerate_sizes(kind, dt):
    """A batch of one sample, towers of two features, a single flat output (and a single
    per-feature output / a single cross layer): every padded operand is almost all padding."""
    w = wl.scaled(wl.mid(), max_rows=200, batch=1, num_tables=4)
    w.table_to_tower = [0, 0, 1, 1]
    w.tm_kind = kind
    w.tm_out = [1, 1]
    w.tm_cross_layers = 1 if kind == "cross_linear" else 0
    if kind == "dlrm":
        w.tm_feat_out = 1
        w.tm_out = [1 + 2 * 1] * 2
    w.tm_dtype = dt
    w.pooled_dtype = dt
    check_tm_bwd(w, rtol=(4e-2 if kind == "cross_linear" else 2e-2) if dt != "f32" else 1e-4)


@pytest.mark.parametrize("D", [64, 32, 16, 8])
def test_compression_ratios_of_the_cross_module(D):
    """The DCN Tower Module at the output widths of the paper's compression study (Table 5):
    O = |F| D for D = 64 ... 8 with |F| = 4 features of N = 128, i.e. CR = D / N from 1/2 down to
    1/16; forward (training variant) and backward."""
    w = wl.scaled(wl.large(), max_rows=300, batch=97, num_tables=4)
    w.table_to_tower = [0, 0, 0, 0]
    w.dims = [128] * 4
    w.tm_out = [4 * D]
    w.tm_cross_layers = 2
    dw = DeviceWorkload(w)
    tm = TowerModules(dw)
    idx, off = wl.lookup_batch(w)
    pooled = oracle.lookup_towered(dw.host_tables, w.table_dtype, w.dims, w.table_to_tower, idx, off, w.batch)
    enc = oracle.round_to(pooled[0], tm.dtype)
    y = to_f64(tm.run(to_device(enc, tm.dtype).reshape(-1))).reshape(w.batch, 4 * D)
    ref = tm.oracle([wl.decode(enc, tm.dtype)])[0]
    assert_close(y, wl.decode(oracle.round_to(ref, tm.dtype), tm.dtype), RTOL[tm.dtype], "cross module, D = %d" % D)
    check_tm_bwd(w, rtol=4e-2, keep=True)


@pytest.mark.parametrize("keep", [False, True])
@pytest.mark.parametrize("dt,rank", [("bf16", 64), ("bf16", 256), ("f16", 32), ("f32", 5)])
def test_lowrank_cross_module(dt, rank, keep):
    """Two low-rank DCN-v2 cross layers on 512-wide towers, then 512 -> 96; batch 150; with the
    backward recomputing u_l and x_l, and on what the training forward kept."""
    w = wl.scaled(wl.large(), max_rows=300, batch=150, num_tables=8)
    w.table_to_tower = [0, 0, 0, 0, 1, 1, 1, 1]
    w.tm_out = [96, 96]
    w.tm_kind = wl.TM_CROSS_LOWRANK_LINEAR
    w.tm_cross_layers = 2
    w.tm_feat_out = rank
    w.tm_dtype = dt
    w.pooled_dtype = dt
    check_tm_bwd(w, rtol=1e-4 if dt == "f32" else 4e-2, keep=keep)


def _random_tower_config(seed):
    """A seeded, arbitrary small configuration: two towers of 1-5 features each, any module
    kind, ragged batch and output widths, every dtype (table dims a multiple of 8 so that the
    16-bit types accept them)."""
    rng = np.random.default_rng(1000 + seed)
    kinds = [wl.TM_LINEAR, wl.TM_LINEAR_RELU, wl.TM_DOT_LINEAR, wl.TM_CROSS_LINEAR, wl.TM_DLRM,
             wl.TM_CROSS_LOWRANK_LINEAR]
    kind = kinds[seed % len(kinds)]
    dt = ["bf16", "f16", "f32"][(seed // len(kinds)) % 3]
    nfs = [int(rng.integers(1, 6)), int(rng.integers(1, 6))]
    dims = [int(rng.choice([8, 16, 32, 64, 128])), int(rng.choice([8, 16, 32, 64, 128]))]
    w = wl.scaled(wl.mid(), max_rows=200, batch=int(rng.integers(1, 700)), num_tables=sum(nfs))
    w.table_to_tower = [0] * nfs[0] + [1] * nfs[1]
    w.dims = [dims[0]] * nfs[0] + [dims[1]] * nfs[1]
    w.tm_kind = kind
    w.tm_dtype = w.pooled_dtype = dt
    w.tm_cross_layers = int(rng.integers(1, 3)) if kind in (wl.TM_CROSS_LINEAR, wl.TM_CROSS_LOWRANK_LINEAR) else 0
    w.tm_out = [int(rng.integers(1, 300)), int(rng.integers(1, 300))]
    if kind == wl.TM_DLRM:
        w.tm_feat_out = int(rng.integers(1, 40))
        w.tm_out = [int(rng.integers(1, 200)) + nf * w.tm_feat_out for nf in nfs]
    if kind == wl.TM_CROSS_LOWRANK_LINEAR:
        w.tm_feat_out = int(rng.integers(1, 12)) * 8 if dt != "f32" else int(rng.integers(1, 70))
    return w


@pytest.mark.parametrize("seed", range(36))
def test_random_small_configurations(seed):
    """Forward (plain and training variant, bit-identical) and backward of arbitrary small towers
    against the oracle: odd widths, one-sample batches, single-feature towers, every kind and
    dtype; what the hand-picked cases above do not happen to hit."""
    w = _random_tower_config(seed)
    dw = DeviceWorkload(w)
    tm = TowerModules(dw)
    idx, off = wl.lookup_batch(w)
    pooled = oracle.lookup_towered(dw.host_tables, w.table_dtype, w.dims, w.table_to_tower, idx, off, w.batch)
    enc = [oracle.round_to(p, tm.dtype) for p in pooled]
    x_dev = torch.cat([to_device(e, tm.dtype).reshape(-1) for e in enc])
    got = to_f64(tm.run(x_dev))
    ref = tm.oracle([wl.decode(e, tm.dtype) for e in enc])
    deep = w.tm_cross_layers > 0
    ftol = (1e-4 if deep else 1e-5) if tm.dtype == "f32" else (4e-2 if deep else 2e-2)
    for t, (g, r) in enumerate(zip(dw.split_towers(got, tm.out_widths), ref)):
        if tm.dtype != "f32":
            r = wl.decode(oracle.round_to(r, tm.dtype), tm.dtype)
        assert_close(g, r, ftol, "seed %d %s forward tower %d" % (seed, w.tm_kind, t))
    check_tm_bwd(w, rtol=ftol, keep=True)


def _random_medium_config(seed):
    """Larger arbitrary towers: 2-16 features of 32-128 columns, batches and widths that are
    sometimes whole multiples of the 256 x 256 tile (the contraction then loads its operand
    tiles straight into LDS) and sometimes ragged."""
    rng = np.random.default_rng(5000 + seed)
    kinds = [wl.TM_LINEAR_RELU, wl.TM_DOT_LINEAR, wl.TM_CROSS_LINEAR, wl.TM_DLRM, wl.TM_CROSS_LOWRANK_LINEAR]
    kind = kinds[seed % len(kinds)]
    dt = ["bf16", "f16"][(seed // len(kinds)) % 2]
    nfs = [int(rng.choice([2, 4, 8, 16])), int(rng.integers(2, 13))]
    dims = [int(rng.choice([64, 128])), int(rng.choice([32, 64, 128]))]
    batch = int(rng.choice([256, 512, 768, 1024])) if rng.random() < 0.5 else int(rng.integers(200, 1500))
    w = wl.scaled(wl.mid(), max_rows=300, batch=batch, num_tables=sum(nfs))
    w.table_to_tower = [0] * nfs[0] + [1] * nfs[1]
    w.dims = [dims[0]] * nfs[0] + [dims[1]] * nfs[1]
    w.tm_kind = kind
    w.tm_dtype = w.pooled_dtype = dt
    w.tm_cross_layers = int(rng.integers(1, 3)) if kind in (wl.TM_CROSS_LINEAR, wl.TM_CROSS_LOWRANK_LINEAR) else 0
    w.tm_out = [int(rng.choice([256, 512])) if rng.random() < 0.5 else int(rng.integers(100, 600)) for _ in nfs]
    if kind == wl.TM_DLRM:
        w.tm_feat_out = int(rng.integers(1, 5)) * 8
        w.tm_out = [int(rng.integers(100, 400)) + nf * w.tm_feat_out for nf in nfs]
    if kind == wl.TM_CROSS_LOWRANK_LINEAR:
        w.tm_feat_out = int(rng.choice([64, 128, 256]))
    return w


@pytest.mark.parametrize("seed", range(20))
def test_random_medium_configurations(seed):
    """Forward and backward of arbitrary towers wide and long enough for the 256 x 256 kernel,
    the in-kernel dot terms, split-K weight gradients and the straight-to-LDS operand loads."""
    w = _random_medium_config(seed)
    dw = DeviceWorkload(w)
    tm = TowerModules(dw)
    idx, off = wl.lookup_batch(w)
    pooled = oracle.lookup_towered(dw.host_tables, w.table_dtype, w.dims, w.table_to_tower, idx, off, w.batch)
    enc = [oracle.round_to(p, tm.dtype) for p in pooled]
    x_dev = torch.cat([to_device(e, tm.dtype).reshape(-1) for e in enc])
    got = to_f64(tm.run(x_dev))
    ref = tm.oracle([wl.decode(e, tm.dtype) for e in enc])
    ftol = 4e-2 if w.tm_cross_layers > 0 else 2e-2
    for t, (g, r) in enumerate(zip(dw.split_towers(got, tm.out_widths), ref)):
        r = wl.decode(oracle.round_to(r, tm.dtype), tm.dtype)
        assert_close(g, r, ftol, "seed %d %s forward tower %d" % (seed, w.tm_kind, t))
    check_tm_bwd(w, rtol=ftol, keep=bool(seed & 1))


@pytest.mark.parametrize("switch", ["DMT_TM_BIG=0", "DMT_TM_FUSE=0", "DMT_TMB_KSPLIT=3", "DMT_TM_DIRECT=0"])
@pytest.mark.parametrize("seed", range(10))
def test_random_medium_configurations_on_the_other_kernel_choices(seed, switch, monkeypatch):
    """The same towers with one of the plan's kernel choices turned the other way."""
    name, value = switch.split("=")
    monkeypatch.setenv(name, value)
    w = _random_medium_config(seed)
    check_tm_bwd(w, rtol=4e-2 if w.tm_cross_layers > 0 else 2e-2, keep=bool(seed & 1))


def test_rejects_bad_arguments():
    w = wl.tiny()
    dw = DeviceWorkload(w)
    tm = TowerModules(dw)
    dmt = dw.dmt
    x = torch.zeros(w.batch * sum(w.tower_widths()), dtype=torch.float32, device="cuda")
    dy = torch.zeros(w.batch * sum(w.tm_out), dtype=torch.float32, device="cuda")
    dx = torch.zeros_like(x)
    g = [dict(dw_proj=torch.zeros(o, k, device="cuda"), db_proj=torch.zeros(o, device="cuda"))
         for o, k in zip(w.tm_out, w.tm_in_dims())]
    arr = dmt.make_tm_grads(g)
    small = torch.empty(32, dtype=torch.int64, device="cuda")
    with pytest.raises(dmt.DmtError) as e:       # workspace too small
        dmt.dmt_tower_module_bwd(dw.plan, tm.params, x, x, w.batch, dy, dx, arr, small)
    assert e.value.code == dmt.binding.DMT_ENOMEM
    big = torch.empty(dmt.dmt_tm_bwd_workspace_bytes(dw.plan, tm.params, w.batch) // 8 + 32,
                      dtype=torch.int64, device="cuda")
    with pytest.raises(dmt.DmtError) as e:       # a ReLU tower needs the forward's output
        dmt.dmt_tower_module_bwd(dw.plan, tm.params, x, None, w.batch, dy, dx, arr, big)
    assert e.value.code == dmt.binding.DMT_EINVAL
    torch.cuda.synchronize()


@pytest.mark.parametrize("which", ["tiny_f32", "mid_bf16"])
def test_whole_tower_step_chains_into_the_sparse_update(which):
    """lookup -> Tower Module -> (gradient of the module outputs) -> Tower Module backward ->
    sorted segment-reduce + rowwise Adagrad, every stage fed by the previous one on the GPU,
    against the same chain of oracles: the sparse update receives dL/d(pooled) as the module's
    backward produced it."""
    if which == "tiny_f32":
        w, rtol = wl.tiny(), 1e-4
    else:
        w, rtol = wl.scaled(wl.mid(True), max_rows=20000, batch=301, num_tables=16), 3e-2
    dw = DeviceWorkload(w, with_state=True)
    tm = TowerModules(dw)
    dmt = dw.dmt
    B = w.batch
    idx, off = wl.lookup_batch(w)
    tables0 = [t.copy() for t in dw.host_tables]
    st0 = [np.zeros(r, dtype=np.float32) for r in w.rows]
    # GPU chain
    x_dev = dw.lookup(idx, off, tm.dtype)
    y_dev = tm.run(x_dev)
    dy = wl.grad_tm_out(w)
    if w.tm_kind == wl.TM_LINEAR_RELU:
        pooled = oracle.lookup_towered(tables0, w.table_dtype, w.dims, w.table_to_tower, idx, off, B)
        o = 0
        for t in range(w.num_towers):
            x64 = wl.decode(oracle.round_to(pooled[t], tm.dtype), tm.dtype)
            pre = oracle.tm_linear(x64, tm.dec[t]["w_proj"], tm.dec[t]["b_proj"])
            near = np.abs(pre) < 1e-3 * np.sqrt(np.mean(pre * pre))
            dy[o:o + B * w.tm_out[t]].reshape(B, -1)[near] = 0.0
            o += B * w.tm_out[t]
    got_dx, _ = run_bwd(dw, tm, x_dev, y_dev, torch.from_numpy(dy).cuda())
    d_idx, d_off = torch.from_numpy(idx).cuda(), torch.from_numpy(off).cuda()
    ws = torch.empty(max(dmt.dmt_bwd_workspace_bytes(dw.plan, B, len(idx)), 256) // 8 + 32,
                     dtype=torch.int64, device="cuda")
    dx_dev = torch.from_numpy(got_dx.astype(np.float32)).cuda()
    dmt.dmt_tower_lookup_bwd_update(dw.plan, d_idx, d_off, B, dx_dev, w.lr, w.eps, ws)
    torch.cuda.synchronize()
    assert dmt.dmt_last_device_error(dw.plan) == -1
    # oracle chain
    pooled = oracle.lookup_towered(tables0, w.table_dtype, w.dims, w.table_to_tower, idx, off, B)
    tables_of = w.tower_tables()
    ref_dx, o = [], 0
    for t in range(w.num_towers):
        x64 = wl.decode(oracle.round_to(pooled[t], tm.dtype), tm.dtype)
        d = tm.dec[t]
        dyt = dy[o:o + B * w.tm_out[t]].reshape(B, w.tm_out[t])
        o += B * w.tm_out[t]
        if w.tm_kind == wl.TM_DOT_LINEAR:
            dx = tm_bwd.tm_dot_linear_bwd(x64, len(tables_of[t]), d["w_proj"], d["b_proj"], dyt)[0]
        else:
            dx = tm_bwd.tm_linear_bwd(x64, d["w_proj"], d["b_proj"], dyt,
                                      relu=w.tm_kind == wl.TM_LINEAR_RELU)[0]
        ref_dx.append(dx.astype(np.float32).reshape(-1))
    ref = oracle.bwd_update(tables0, w.table_dtype, st0, w.dims, w.table_to_tower, idx, off, B,
                            np.concatenate(ref_dx), w.lr, w.eps)
    for f in range(w.num_tables):
        m = ref["key_table"] == f
        rows = ref["key_row"][m]
        if not len(rows):
            continue
        sel = torch.from_numpy(rows).cuda()
        want = ref["new_rows"][m][:, :w.dims[f]]
        if w.table_dtype != "f32":
            want = wl.decode(oracle.round_to(want, w.table_dtype), w.table_dtype)
        assert_close(to_f64(dw.tables[f][sel]), want, max(rtol, RTOL[w.table_dtype]),
                     "%s chained rows of table %d" % (w.name, f))
        assert_close(to_f64(dw.states[f][sel]), ref["new_state"][m].astype(np.float32), rtol,
                     "%s chained state of table %d" % (w.name, f))
