"""The C-ABI library loads, exports every symbol include/dmt.h declares, and its
host-side validation rejects bad arguments before touching any device (CPU only)."""
import ctypes
import os
import re

import pytest

import paper_2403_00877_amd as dmt
from paper_2403_00877_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "dmt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dmt_[a-z_0-9]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    lib = ctypes.CDLL(dmt.library_path())
    names = _declared_symbols()
    assert {"dmt_tower_lookup_fwd", "dmt_tower_module_fwd", "dmt_tower_lookup_bwd_update"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names


def test_status_strings():
    assert [dmt.status_str(i) for i in range(6)] == [
        "DMT_OK", "DMT_EINVAL", "DMT_ENOTSUP", "DMT_EBOUNDS", "DMT_ENOMEM", "DMT_EHIP"]
    assert dmt.dmt_kernel_name(0) == "lookup_fwd" and dmt.dmt_kernel_name(99) == "?"


def test_plan_layout_matches_reference():
    rows, dims, t2t = [10, 20, 30, 40, 50], [8, 16, 8, 32, 16], [1, 0, 1, 0, 2]
    p = dmt.dmt_plan_create(rows, dims, "f16", 3, t2t, 7, 100)
    base, width, col = dmt.dmt_plan_layout(p, 7)
    assert width == [48, 16, 16]
    assert base == [0, 7 * 48, 7 * 64, 7 * 80]
    assert col == [0, 0, 8, 16, 0]
    assert dmt.dmt_plan_layout(p, 3)[0] == [0, 144, 192, 240]


@pytest.mark.parametrize("kwargs,code", [
    (dict(dims=[7, 8]), binding.DMT_ENOTSUP),                 # 14-byte rows
    (dict(dims=[1024, 8]), binding.DMT_ENOTSUP),              # 2 KB rows
    (dict(rows=[0, 5]), binding.DMT_EINVAL),
    (dict(t2t=[0, 2]), binding.DMT_EINVAL),                   # tower id out of range
    (dict(t2t=[1, 1]), binding.DMT_EINVAL),                   # tower 0 empty
    (dict(max_batch=0), binding.DMT_EINVAL),
    (dict(max_nnz=1 << 31), binding.DMT_ENOTSUP),
    (dict(rows=[1 << 31, 5]), binding.DMT_ENOTSUP),
])
def test_plan_create_rejects(kwargs, code):
    a = dict(rows=[5, 5], dims=[8, 8], t2t=[0, 1], max_batch=4, max_nnz=64)
    a.update(kwargs)
    with pytest.raises(dmt.DmtError) as e:
        dmt.dmt_plan_create(a["rows"], a["dims"], "f16", 2, a["t2t"], a["max_batch"], a["max_nnz"])
    assert e.value.code == code


def test_hot_calls_validate_before_launching():
    """Null pointers, unbound plans and oversize batches come back as error codes
    from the host checks (this container has no GPU, so nothing may launch)."""
    lib = ctypes.CDLL(dmt.library_path())
    p = dmt.dmt_plan_create([5, 5], [8, 8], "f16", 2, [0, 1], 4, 64)
    vp = ctypes.c_void_p
    i64 = ctypes.c_int64
    fwd = lib.dmt_tower_lookup_fwd
    fwd.argtypes = [vp, vp, vp, i64, i64, vp, ctypes.c_int, vp]
    fake = vp(4096)
    assert fwd(None, fake, fake, 4, 8, fake, 1, None) == binding.DMT_EINVAL
    assert fwd(p.handle, fake, None, 4, 8, fake, 1, None) == binding.DMT_EINVAL
    assert fwd(p.handle, fake, fake, 5, 8, fake, 1, None) == binding.DMT_EINVAL        # B > max_batch
    assert fwd(p.handle, fake, fake, 4, 65, fake, 1, None) == binding.DMT_EINVAL       # nnz > max_nnz
    assert fwd(p.handle, fake, fake, 4, 8, vp(4100), 1, None) == binding.DMT_EINVAL    # misaligned out
    assert fwd(p.handle, fake, fake, 4, 8, fake, 7, None) == binding.DMT_EINVAL        # bad dtype
    assert fwd(p.handle, fake, fake, 4, 8, fake, 1, None) == binding.DMT_EINVAL        # plan not bound
    bwd = lib.dmt_tower_lookup_bwd_update
    bwd.argtypes = [vp, vp, vp, i64, i64, vp, ctypes.c_float, ctypes.c_float, vp, ctypes.c_size_t, vp, vp]
    assert bwd(p.handle, fake, fake, 4, 8, fake, 0.01, 1e-8, fake, 1 << 20, None, None) == binding.DMT_EINVAL
    tm = lib.dmt_tower_module_fwd
    tm.argtypes = [vp, vp, vp, i64, vp, ctypes.c_int, vp, ctypes.c_size_t, vp]
    params = dmt.binding.dmt_tm_params * 2
    arr = params()
    assert tm(p.handle, arr, fake, 4, fake, 2, None, 0, None) == binding.DMT_EINVAL     # null weights
    arr[0].kind = arr[1].kind = 3
    arr[0].out_dim = arr[1].out_dim = 8
    arr[0].w_proj = arr[1].w_proj = 4096
    arr[0].b_proj = arr[1].b_proj = 4096
    assert tm(p.handle, arr, fake, 4, fake, 2, None, 0, None) == binding.DMT_EINVAL     # cross without layers
    # workspace sizing is pure host arithmetic
    assert dmt.dmt_bwd_workspace_bytes(p, 4, 64) > 2 * 8 * 64
    arr[0].kind = arr[1].kind = 2
    need = lib.dmt_tm_workspace_bytes
    need.restype = ctypes.c_size_t
    need.argtypes = [vp, vp, i64]
    assert need(p.handle, arr, 4) > 0                    # dot terms + repacked weights
    arr[0].kind = arr[1].kind = 0
    assert need(p.handle, arr, 4) == 0
    ws = ctypes.c_void_p(4096)
    arr[0].kind = arr[1].kind = 2
    assert tm(p.handle, arr, fake, 4, fake, 2, ws, 16, None) == binding.DMT_ENOMEM      # workspace too small


def test_tower_module_backward_and_keep_validate_on_the_host():
    """dmt_tower_module_bwd / _fwd_keep: sizes are host arithmetic, bad arguments come back as
    codes before anything is launched."""
    lib = ctypes.CDLL(dmt.library_path())
    vp, i64, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_size_t
    # two towers of two 8-wide tables each, batch up to 4
    p = dmt.dmt_plan_create([5, 5, 5, 5], [8, 8, 8, 8], "f16", 2, [0, 0, 1, 1], 4, 64)
    arr = (dmt.binding.dmt_tm_params * 2)()
    for a in arr:
        a.kind, a.out_dim, a.w_proj, a.b_proj = binding.DMT_TM_CROSS_LINEAR, 8, 4096, 4096
        a.num_cross_layers = 2
        for l in range(2):
            a.w_cross[l] = a.b_cross[l] = 4096
    # kept: per tower and layer x_{l+1} and u_l, each B * 16 f16 values rounded up to 256 bytes
    assert dmt.dmt_tm_kept_bytes(p, arr, 4, "f16") == 2 * 2 * 2 * 256
    assert dmt.dmt_tm_kept_bytes(p, arr, 4, "f32") == 2 * 2 * 2 * 256
    assert dmt.dmt_tm_kept_bytes(p, arr, 3, "bf16") == 2 * 2 * 2 * 256
    need = dmt.dmt_tm_bwd_workspace_bytes(p, arr, 4)
    assert need > 0 and dmt.dmt_tm_bwd_workspace_bytes(p, arr, 2) <= need
    for a in arr:
        a.kind = binding.DMT_TM_DOT_LINEAR
    # dot towers keep their dot terms (1 term padded to 8 per sample) and the repacked weights
    # ([8][8 + 16] f16 = 384 bytes), each rounded up to 256 bytes
    assert dmt.dmt_tm_kept_bytes(p, arr, 4, "f16") == 2 * (256 + 512)
    for a in arr:
        a.kind = binding.DMT_TM_LINEAR
    assert dmt.dmt_tm_kept_bytes(p, arr, 4, "f16") == 0          # linear towers keep nothing
    for a in arr:
        a.kind = binding.DMT_TM_DOT_LINEAR
    grads = (dmt.binding.dmt_tm_grads * 2)()
    bwd = lib.dmt_tower_module_bwd
    bwd.argtypes = [vp, vp, vp, vp, i64, vp, ctypes.c_int, vp, vp, vp, sz, vp, sz, vp]
    fake = vp(4096)
    args = lambda **kw: [kw.get("plan", p.handle), arr, kw.get("pooled", fake), fake, kw.get("B", 4), fake, 1,
                         kw.get("dx", fake), grads, kw.get("kept", None), kw.get("kept_bytes", 0),
                         kw.get("ws", fake), kw.get("ws_bytes", 1 << 30), None]
    assert bwd(*args()) == binding.DMT_EINVAL                     # gradient outputs not given
    for g in grads:
        g.dw_proj = g.db_proj = 4096
    assert bwd(*args(plan=None)) == binding.DMT_EINVAL
    assert bwd(*args(pooled=None)) == binding.DMT_EINVAL
    assert bwd(*args(B=5)) == binding.DMT_EINVAL                  # B > max_batch
    assert bwd(*args(dx=vp(4100))) == binding.DMT_EINVAL          # misaligned output
    assert bwd(*args(ws=vp(4100))) == binding.DMT_EINVAL          # misaligned workspace
    assert bwd(*args(ws_bytes=64)) == binding.DMT_ENOMEM
    for a in arr:
        a.kind = binding.DMT_TM_CROSS_LINEAR
    assert bwd(*args()) == binding.DMT_EINVAL                     # cross gradients not given
    for g in grads:
        for l in range(2):
            g.dw_cross[l] = g.db_cross[l] = 4096
    assert bwd(*args(kept=fake, kept_bytes=64)) == binding.DMT_ENOMEM
    assert bwd(*args(kept=vp(4100), kept_bytes=1 << 20)) == binding.DMT_EINVAL
    keep = lib.dmt_tower_module_fwd_keep
    keep.argtypes = [vp, vp, vp, i64, vp, ctypes.c_int, vp, sz, vp, sz, vp]
    assert keep(p.handle, arr, fake, 4, fake, 1, None, 0, fake, 1 << 20, None) == binding.DMT_EINVAL
    assert keep(p.handle, arr, fake, 4, fake, 1, fake, 64, fake, 1 << 20, None) == binding.DMT_ENOMEM
    # a DLRM tower needs at least one flat output beside its per-feature ones
    for a in arr:
        a.kind, a.feat_out, a.out_dim = binding.DMT_TM_DLRM, 4, 8      # 2 features * 4 = all 8 outputs
    assert bwd(*args()) == binding.DMT_EINVAL
    assert dmt.dmt_tm_bwd_workspace_bytes(p, arr, 4) == 0
    for a in arr:
        a.out_dim = 9
    assert dmt.dmt_tm_bwd_workspace_bytes(p, arr, 4) > 0


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True)
    assert r.returncode != 0 and "ONE GPU" in r.stderr


def test_sptt_peer_order_matches_the_papers_example_and_the_oracle():
    from oracle import sptt
    assert dmt.dmt_sptt_peer_order(4, 2) == [0, 2, 1, 3]          # Sec. 3.1.1's example
    for G, L in ((8, 4), (8, 2), (16, 8), (6, 3), (5, 1), (4, 4), (1, 1)):
        assert dmt.dmt_sptt_peer_order(G, L) == sptt.peer_order(G, L)
    order = (ctypes.c_int32 * 8)()
    raw = dmt.binding._lib.dmt_sptt_peer_order
    assert raw(8, 3, order) == 1 and raw(0, 1, order) == 1 and raw(8, 0, order) == 1 and raw(8, 2, None) == 1
