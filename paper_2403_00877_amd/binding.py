"""ctypes binding of libdmt.so: argument marshalling only.

Every function here has the name of the C entry point it calls (include/dmt.h)
and does nothing but turn torch tensors into pointers and sizes.  All
arithmetic of the path runs in the library's HIP kernels.  There is no
fallback: if the library cannot be loaded the import of this module raises.
"""
from __future__ import annotations

import ctypes
from typing import List, Optional, Sequence

import torch

from . import build as _build

DMT_OK, DMT_EINVAL, DMT_ENOTSUP, DMT_EBOUNDS, DMT_ENOMEM, DMT_EHIP = range(6)
DMT_F32, DMT_F16, DMT_BF16 = 0, 1, 2
DMT_TM_LINEAR, DMT_TM_LINEAR_RELU, DMT_TM_DOT_LINEAR, DMT_TM_CROSS_LINEAR, DMT_TM_DLRM = 0, 1, 2, 3, 4
DMT_TM_CROSS_LOWRANK_LINEAR = 5
DMT_MAX_CROSS_LAYERS = 4

DTYPE_CODE = {"f32": DMT_F32, "f16": DMT_F16, "bf16": DMT_BF16,
              torch.float32: DMT_F32, torch.float16: DMT_F16, torch.bfloat16: DMT_BF16}
TORCH_DTYPE = {DMT_F32: torch.float32, DMT_F16: torch.float16, DMT_BF16: torch.bfloat16}
TM_KIND_CODE = {"linear": DMT_TM_LINEAR, "linear_relu": DMT_TM_LINEAR_RELU,
                "dot_linear": DMT_TM_DOT_LINEAR, "cross_linear": DMT_TM_CROSS_LINEAR,
                "dlrm": DMT_TM_DLRM, "cross_lowrank_linear": DMT_TM_CROSS_LOWRANK_LINEAR}


class dmt_tm_params(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("out_dim", ctypes.c_int32),
                ("num_cross_layers", ctypes.c_int32), ("feat_out", ctypes.c_int32),
                ("w_proj", ctypes.c_void_p), ("b_proj", ctypes.c_void_p),
                ("w_cross", ctypes.c_void_p * DMT_MAX_CROSS_LAYERS),
                ("b_cross", ctypes.c_void_p * DMT_MAX_CROSS_LAYERS)]


class dmt_tm_grads(ctypes.Structure):
    _fields_ = [("dw_proj", ctypes.c_void_p), ("db_proj", ctypes.c_void_p),
                ("dw_cross", ctypes.c_void_p * DMT_MAX_CROSS_LAYERS),
                ("db_cross", ctypes.c_void_p * DMT_MAX_CROSS_LAYERS)]


class dmt_bwd_debug(ctypes.Structure):
    _fields_ = [("sorted_keys", ctypes.c_void_p), ("sorted_bag", ctypes.c_void_p),
                ("unique_keys", ctypes.c_void_p), ("seg_off", ctypes.c_void_p),
                ("num_unique", ctypes.c_void_p)]


class DmtError(RuntimeError):
    def __init__(self, where: str, code: int):
        self.code = code
        super().__init__("%s failed: %s" % (where, status_str(code)))


def _load() -> ctypes.CDLL:
    if _build.is_stale():
        # missing, or built from other sources than the tree holds: results would describe code
        # that is no longer there
        import sys
        print("[dmt] %s is missing or stale: building it from the sources in the tree" % _build.LIB,
              file=sys.stderr, flush=True)
        _build.build()          # raises if hipcc is missing or the build fails
    lib = ctypes.CDLL(_build.LIB)
    vp, i32, i64, f32, sz = (ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_float,
                             ctypes.c_size_t)
    lib.dmt_status_str.restype = ctypes.c_char_p
    lib.dmt_status_str.argtypes = [ctypes.c_int]
    lib.dmt_plan_create.argtypes = [ctypes.POINTER(vp), i32, vp, vp, ctypes.c_int, i32, vp, i64, i64]
    lib.dmt_plan_destroy.argtypes = [vp]
    lib.dmt_plan_destroy.restype = None
    lib.dmt_plan_layout.argtypes = [vp, i64, vp, vp, vp]
    lib.dmt_plan_bind.argtypes = [vp, vp, vp]
    lib.dmt_tower_lookup_fwd.argtypes = [vp, vp, vp, i64, i64, vp, ctypes.c_int, vp]
    lib.dmt_tm_workspace_bytes.argtypes = [vp, vp, i64]
    lib.dmt_tm_workspace_bytes.restype = sz
    lib.dmt_tower_module_fwd.argtypes = [vp, vp, vp, i64, vp, ctypes.c_int, vp, sz, vp]
    lib.dmt_tm_bwd_workspace_bytes.argtypes = [vp, vp, i64]
    lib.dmt_tm_bwd_workspace_bytes.restype = sz
    lib.dmt_tower_module_bwd.argtypes = [vp, vp, vp, vp, i64, vp, ctypes.c_int, vp, vp, vp, sz, vp, sz, vp]
    lib.dmt_tm_kept_bytes.argtypes = [vp, vp, i64, ctypes.c_int]
    lib.dmt_tm_kept_bytes.restype = sz
    lib.dmt_tower_module_fwd_keep.argtypes = [vp, vp, vp, i64, vp, ctypes.c_int, vp, sz, vp, sz, vp]
    lib.dmt_bwd_workspace_bytes.argtypes = [vp, i64, i64]
    lib.dmt_bwd_workspace_bytes.restype = sz
    lib.dmt_tower_lookup_bwd_update.argtypes = [vp, vp, vp, i64, i64, vp, f32, f32, vp, sz, vp, vp]
    lib.dmt_bwd_noalloc_scratch_bytes.argtypes = []
    lib.dmt_bwd_noalloc_scratch_bytes.restype = sz
    lib.dmt_tower_lookup_bwd_update_noalloc.argtypes = [vp, vp, vp, i64, i64, vp, f32, f32, vp]
    lib.dmt_last_device_error.argtypes = [vp, vp, ctypes.POINTER(i64)]
    lib.dmt_kernel_name.restype = ctypes.c_char_p
    lib.dmt_kernel_name.argtypes = [i32]
    lib.dmt_profile_enable.argtypes = [vp, ctypes.c_uint32]
    lib.dmt_profile_read.argtypes = [vp, vp, vp, vp]
    lib.dmt_calibration_copy.argtypes = [vp, vp, sz, vp]
    lib.dmt_calibration_gather.argtypes = [vp, ctypes.c_int64, ctypes.c_int32, vp, ctypes.c_int64, vp, vp]
    f64 = ctypes.c_double
    lib.dmt_tp_workspace_bytes.argtypes = [vp, i64]
    lib.dmt_tp_workspace_bytes.restype = sz
    lib.dmt_tp_interaction.argtypes = [vp, vp, i64, ctypes.c_int, vp, vp, sz, vp]
    lib.dmt_tp_embed.argtypes = [vp, i32, ctypes.c_int, i32, i32, f64, vp, vp, ctypes.POINTER(f64)]
    lib.dmt_tp_kmeans.argtypes = [vp, i32, i32, i32, f64, vp, i32, vp, vp, ctypes.POINTER(i32)]
    lib.dmt_plan_set_row_shards.argtypes = [vp, vp]
    lib.dmt_sptt_peer_order.argtypes = [i32, i32, vp]
    lib.dmt_sptt_peer_permute.argtypes = [vp, vp, i64, i32, i32, i64, vp]
    lib.dmt_sptt_shuffle.argtypes = [vp, vp, i64, i64, i64, vp]
    lib.dmt_sptt_peer_permute_ids.argtypes = [vp, vp, i64, i32, i32, i64, i64, vp, vp, vp]
    return lib


_lib = _load()

EXPORTS = ["dmt_status_str", "dmt_plan_create", "dmt_plan_destroy", "dmt_plan_layout",
           "dmt_plan_bind", "dmt_tower_lookup_fwd", "dmt_tm_workspace_bytes",
           "dmt_tower_module_fwd", "dmt_tm_bwd_workspace_bytes", "dmt_tower_module_bwd",
           "dmt_tm_kept_bytes", "dmt_tower_module_fwd_keep",
           "dmt_bwd_workspace_bytes", "dmt_tower_lookup_bwd_update",
           "dmt_last_device_error", "dmt_kernel_name", "dmt_profile_enable", "dmt_profile_read",
           "dmt_calibration_copy", "dmt_calibration_gather", "dmt_tp_workspace_bytes", "dmt_tp_interaction",
           "dmt_tp_embed", "dmt_tp_kmeans", "dmt_sptt_peer_order", "dmt_sptt_peer_permute",
           "dmt_sptt_shuffle", "dmt_plan_set_row_shards", "dmt_bwd_noalloc_scratch_bytes",
           "dmt_tower_lookup_bwd_update_noalloc", "dmt_sptt_peer_permute_ids"]

DMT_K_COUNT = 15
TP_STRATEGY_CODE = {"diverse": 0, "coherent": 1}


def library_path() -> str:
    return _build.LIB


def status_str(code: int) -> str:
    return _lib.dmt_status_str(int(code)).decode()


def _check(where: str, code: int) -> None:
    if code != DMT_OK:
        raise DmtError(where, code)


def _stream(stream) -> Optional[int]:
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream))


def _ptr(t: Optional[torch.Tensor]):
    return ctypes.c_void_p(0 if t is None else t.data_ptr())


class dmt_plan:
    """Owner of a C `dmt_plan*`."""

    def __init__(self, rows: Sequence[int], dims: Sequence[int], table_dtype, num_towers: int,
                 table_to_tower: Sequence[int], max_batch: int, max_nnz: int):
        self.num_tables = len(rows)
        self.num_towers = int(num_towers)
        self.table_dtype = DTYPE_CODE[table_dtype]
        r = (ctypes.c_int64 * len(rows))(*rows)
        d = (ctypes.c_int32 * len(dims))(*dims)
        t = (ctypes.c_int32 * len(table_to_tower))(*table_to_tower)
        h = ctypes.c_void_p()
        self._h = None
        _check("dmt_plan_create", _lib.dmt_plan_create(
            ctypes.byref(h), len(rows), r, d, self.table_dtype, num_towers, t, max_batch, max_nnz))
        self._h = h
        self._keep = None

    def __del__(self):
        if getattr(self, "_h", None):
            _lib.dmt_plan_destroy(self._h)
            self._h = None

    @property
    def handle(self):
        return self._h


def dmt_plan_create(rows, dims, table_dtype, num_towers, table_to_tower, max_batch, max_nnz) -> dmt_plan:
    return dmt_plan(rows, dims, table_dtype, num_towers, table_to_tower, max_batch, max_nnz)


def dmt_plan_layout(plan: dmt_plan, B: int):
    """(tower_base [T+1], tower_width [T], col_off [F]) as Python lists."""
    tb = (ctypes.c_int64 * (plan.num_towers + 1))()
    tw = (ctypes.c_int32 * plan.num_towers)()
    co = (ctypes.c_int32 * plan.num_tables)()
    _check("dmt_plan_layout", _lib.dmt_plan_layout(plan.handle, B, tb, tw, co))
    return list(tb), list(tw), list(co)


def dmt_plan_bind(plan: dmt_plan, tables: Sequence[torch.Tensor],
                  adagrad_state: Optional[Sequence[torch.Tensor]] = None) -> None:
    tp = (ctypes.c_void_p * len(tables))(*[t.data_ptr() for t in tables])
    sp = None
    if adagrad_state is not None:
        sp = (ctypes.c_void_p * len(adagrad_state))(*[t.data_ptr() for t in adagrad_state])
    _check("dmt_plan_bind", _lib.dmt_plan_bind(plan.handle, tp, sp))
    plan._keep = (list(tables), None if adagrad_state is None else list(adagrad_state))


def dmt_tower_lookup_fwd(plan: dmt_plan, indices: torch.Tensor, offsets: torch.Tensor, B: int,
                         pooled_out: torch.Tensor, stream=None) -> None:
    _check("dmt_tower_lookup_fwd", _lib.dmt_tower_lookup_fwd(
        plan.handle, _ptr(indices), _ptr(offsets), B, indices.numel(), _ptr(pooled_out),
        DTYPE_CODE[pooled_out.dtype], _stream(stream)))


def make_tm_params(per_tower: Sequence[dict]):
    """per_tower: dicts with kind (str), out_dim, w_proj, b_proj and optionally
    w_cross / b_cross (lists of tensors; for kind "dlrm" the one shared per-feature layer, with
    feat_out its output count).  Returns a ctypes array."""
    arr = (dmt_tm_params * len(per_tower))()
    for a, p in zip(arr, per_tower):
        a.kind = TM_KIND_CODE[p["kind"]]
        a.out_dim = int(p["out_dim"])
        wc = p.get("w_cross") or []
        a.num_cross_layers = len(wc)
        if a.kind == DMT_TM_CROSS_LOWRANK_LINEAR:       # w_cross = [V_0, U_0, V_1, U_1, ...]
            a.num_cross_layers = len(wc) // 2
        a.feat_out = int(p.get("feat_out") or 0)
        a.w_proj = p["w_proj"].data_ptr()
        a.b_proj = p["b_proj"].data_ptr()
        for l, w in enumerate(wc):
            a.w_cross[l] = w.data_ptr()
        for l, b in enumerate(p.get("b_cross") or []):
            a.b_cross[l] = b.data_ptr()
    return arr


def dmt_tm_workspace_bytes(plan: dmt_plan, tm_params, B: int) -> int:
    return int(_lib.dmt_tm_workspace_bytes(plan.handle, tm_params, B))


def dmt_tower_module_fwd(plan: dmt_plan, tm_params, pooled: torch.Tensor, B: int,
                         tm_out: torch.Tensor, workspace: Optional[torch.Tensor] = None,
                         stream=None) -> None:
    _check("dmt_tower_module_fwd", _lib.dmt_tower_module_fwd(
        plan.handle, tm_params, _ptr(pooled), B, _ptr(tm_out), DTYPE_CODE[tm_out.dtype],
        _ptr(workspace), 0 if workspace is None else workspace.numel() * workspace.element_size(),
        _stream(stream)))


def make_tm_grads(per_tower: Sequence[dict]):
    """per_tower: dicts with float32 tensors dw_proj, db_proj and optionally lists
    dw_cross / db_cross.  Returns a ctypes array."""
    arr = (dmt_tm_grads * len(per_tower))()
    for a, g in zip(arr, per_tower):
        a.dw_proj = g["dw_proj"].data_ptr()
        a.db_proj = g["db_proj"].data_ptr()
        for l, w in enumerate(g.get("dw_cross") or []):
            a.dw_cross[l] = w.data_ptr()
        for l, b in enumerate(g.get("db_cross") or []):
            a.db_cross[l] = b.data_ptr()
    return arr


def dmt_tm_bwd_workspace_bytes(plan: dmt_plan, tm_params, B: int) -> int:
    return int(_lib.dmt_tm_bwd_workspace_bytes(plan.handle, tm_params, B))


def _nbytes(t: Optional[torch.Tensor]) -> int:
    return 0 if t is None else t.numel() * t.element_size()


def dmt_tm_kept_bytes(plan: dmt_plan, tm_params, B: int, dtype) -> int:
    return int(_lib.dmt_tm_kept_bytes(plan.handle, tm_params, B, DTYPE_CODE[dtype]))


def dmt_tower_module_fwd_keep(plan: dmt_plan, tm_params, pooled: torch.Tensor, B: int,
                              tm_out: torch.Tensor, kept: Optional[torch.Tensor],
                              workspace: Optional[torch.Tensor] = None, stream=None) -> None:
    _check("dmt_tower_module_fwd_keep", _lib.dmt_tower_module_fwd_keep(
        plan.handle, tm_params, _ptr(pooled), B, _ptr(tm_out), DTYPE_CODE[tm_out.dtype],
        _ptr(kept), _nbytes(kept), _ptr(workspace), _nbytes(workspace), _stream(stream)))


def dmt_tower_module_bwd(plan: dmt_plan, tm_params, pooled: torch.Tensor,
                         tm_out: Optional[torch.Tensor], B: int, grad_tm_out: torch.Tensor,
                         grad_pooled: torch.Tensor, tm_grads, workspace: torch.Tensor,
                         stream=None, kept: Optional[torch.Tensor] = None) -> None:
    assert grad_tm_out.dtype == torch.float32 and grad_pooled.dtype == torch.float32
    _check("dmt_tower_module_bwd", _lib.dmt_tower_module_bwd(
        plan.handle, tm_params, _ptr(pooled), _ptr(tm_out), B, _ptr(grad_tm_out),
        DTYPE_CODE[pooled.dtype], _ptr(grad_pooled), tm_grads, _ptr(kept), _nbytes(kept),
        _ptr(workspace), _nbytes(workspace), _stream(stream)))


def dmt_bwd_workspace_bytes(plan: dmt_plan, B: int, nnz: int) -> int:
    return int(_lib.dmt_bwd_workspace_bytes(plan.handle, B, nnz))


def dmt_tower_lookup_bwd_update(plan: dmt_plan, indices: torch.Tensor, offsets: torch.Tensor,
                                B: int, grad_pooled: torch.Tensor, lr: float, eps: float,
                                workspace: torch.Tensor, stream=None, debug: Optional[dict] = None) -> None:
    dbg = None
    if debug is not None:
        dbg = dmt_bwd_debug()
        for k in ("sorted_keys", "sorted_bag", "unique_keys", "seg_off", "num_unique"):
            setattr(dbg, k, debug[k].data_ptr() if debug.get(k) is not None else None)
        dbg = ctypes.byref(dbg)
    _check("dmt_tower_lookup_bwd_update", _lib.dmt_tower_lookup_bwd_update(
        plan.handle, _ptr(indices), _ptr(offsets), B, indices.numel(), _ptr(grad_pooled),
        lr, eps, _ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream), dbg))


def dmt_bwd_noalloc_scratch_bytes() -> int:
    return int(_lib.dmt_bwd_noalloc_scratch_bytes())


def dmt_tower_lookup_bwd_update_noalloc(plan: dmt_plan, indices: torch.Tensor, offsets: torch.Tensor,
                                        B: int, grad_pooled: torch.Tensor, lr: float, eps: float,
                                        stream=None) -> None:
    _check("dmt_tower_lookup_bwd_update_noalloc", _lib.dmt_tower_lookup_bwd_update_noalloc(
        plan.handle, _ptr(indices), _ptr(offsets), B, indices.numel(), _ptr(grad_pooled),
        lr, eps, _stream(stream)))


def dmt_last_device_error(plan: dmt_plan, stream=None) -> int:
    """-1 when clean, else the smallest position of an id outside its table (and the record is
    cleared).  Raises DmtError(DMT_EINVAL) when the backward found malformed offsets; the
    exception's `position` is the first offending bag."""
    pos = ctypes.c_int64(-1)
    code = _lib.dmt_last_device_error(plan.handle, _stream(stream), ctypes.byref(pos))
    if code not in (DMT_OK, DMT_EBOUNDS):
        e = DmtError("dmt_last_device_error", code)
        e.position = int(pos.value)
        raise e
    return int(pos.value)


def dmt_kernel_name(kernel_id: int) -> str:
    return _lib.dmt_kernel_name(int(kernel_id)).decode()


def dmt_profile_enable(plan: dmt_plan, kernel_mask: int) -> None:
    _check("dmt_profile_enable", _lib.dmt_profile_enable(plan.handle, kernel_mask))


def dmt_profile_read(plan: dmt_plan, stream=None) -> dict:
    """{kernel name: (total_ms, launches)} for the families timed since the last read."""
    ms = (ctypes.c_double * DMT_K_COUNT)()
    n = (ctypes.c_int64 * DMT_K_COUNT)()
    _check("dmt_profile_read", _lib.dmt_profile_read(plan.handle, _stream(stream), ms, n))
    return {dmt_kernel_name(i): (ms[i], n[i]) for i in range(DMT_K_COUNT) if n[i]}


def dmt_calibration_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() >= nbytes
    _check("dmt_calibration_copy", _lib.dmt_calibration_copy(_ptr(dst), _ptr(src), nbytes, _stream(stream)))


DMT_CALIBRATION_GATHER_BLOCKS = 2048


def dmt_calibration_gather(table: torch.Tensor, row_bytes: int, ids: torch.Tensor, out: torch.Tensor,
                           stream=None) -> None:
    """table: any dtype, rows of row_bytes bytes; ids int32; out: at least 2048 * 256 * 16 bytes."""
    rows = table.numel() * table.element_size() // row_bytes
    assert out.numel() * out.element_size() >= DMT_CALIBRATION_GATHER_BLOCKS * 256 * 16
    _check("dmt_calibration_gather", _lib.dmt_calibration_gather(
        _ptr(table), rows, row_bytes, _ptr(ids), ids.numel(), _ptr(out), _stream(stream)))


def dmt_tp_workspace_bytes(plan: dmt_plan, B: int) -> int:
    return int(_lib.dmt_tp_workspace_bytes(plan.handle, B))


def dmt_tp_interaction(plan: dmt_plan, pooled: torch.Tensor, B: int, interaction: torch.Tensor,
                       workspace: torch.Tensor, stream=None) -> None:
    assert interaction.dtype == torch.float32
    assert interaction.numel() >= plan.num_tables * plan.num_tables
    _check("dmt_tp_interaction", _lib.dmt_tp_interaction(
        plan.handle, _ptr(pooled), B, DTYPE_CODE[pooled.dtype], _ptr(interaction),
        _ptr(workspace), _nbytes(workspace), _stream(stream)))


def _host(a, dtype):
    import numpy as np
    return np.ascontiguousarray(a, dtype=dtype)


def dmt_tp_embed(interaction, strategy: str, n: int, steps: int, lr: float, x0):
    """Host arrays in, (coordinates float64 [F][n], stress) out."""
    import numpy as np
    I = _host(interaction, np.float32)
    x0 = _host(x0, np.float64)
    F = I.shape[0]
    assert I.shape == (F, F) and x0.shape == (F, n)
    x = np.empty_like(x0)
    stress = ctypes.c_double(0.0)
    _check("dmt_tp_embed", _lib.dmt_tp_embed(
        I.ctypes.data, F, TP_STRATEGY_CODE[strategy], n, steps, lr, x0.ctypes.data, x.ctypes.data,
        ctypes.byref(stress)))
    return x, float(stress.value)


def dmt_tp_kmeans(x, T: int, ratio: float, centres0, max_iter: int = 100):
    """Host arrays in, (table_to_tower int32 [F], centres float64 [T][n], iterations) out."""
    import numpy as np
    x = _host(x, np.float64)
    c0 = _host(centres0, np.float64)
    F, n = x.shape
    assert c0.shape == (T, n)
    labels = np.empty(F, dtype=np.int32)
    centres = np.empty_like(c0)
    it = ctypes.c_int32(0)
    _check("dmt_tp_kmeans", _lib.dmt_tp_kmeans(
        x.ctypes.data, F, n, T, ratio, c0.ctypes.data, max_iter, labels.ctypes.data,
        centres.ctypes.data, ctypes.byref(it)))
    return labels, centres, int(it.value)


def dmt_sptt_peer_order(G: int, L: int) -> List[int]:
    order = (ctypes.c_int32 * max(G, 1))()
    _check("dmt_sptt_peer_order", _lib.dmt_sptt_peer_order(G, L, order))
    return list(order)


def dmt_sptt_peer_permute(inp: torch.Tensor, out: torch.Tensor, features: int, G: int, L: int,
                          block_bytes: int, stream=None) -> None:
    assert _nbytes(inp) >= features * G * block_bytes and _nbytes(out) >= features * G * block_bytes
    _check("dmt_sptt_peer_permute", _lib.dmt_sptt_peer_permute(
        _ptr(inp), _ptr(out), features, G, L, block_bytes, _stream(stream)))


def dmt_sptt_shuffle(inp: torch.Tensor, out: torch.Tensor, features: int, peers: int,
                     block_bytes: int, stream=None) -> None:
    assert _nbytes(inp) >= features * peers * block_bytes and _nbytes(out) >= features * peers * block_bytes
    _check("dmt_sptt_shuffle", _lib.dmt_sptt_shuffle(
        _ptr(inp), _ptr(out), features, peers, block_bytes, _stream(stream)))


def dmt_sptt_peer_permute_ids(indices: torch.Tensor, offsets: torch.Tensor, features: int, G: int,
                              L: int, B_l: int, out_indices: torch.Tensor, out_offsets: torch.Tensor,
                              stream=None) -> None:
    assert indices.dtype == torch.int32 and offsets.dtype == torch.int64
    assert out_indices.dtype == torch.int32 and out_offsets.dtype == torch.int64
    assert offsets.numel() == features * G * B_l + 1 and out_offsets.numel() >= offsets.numel()
    assert out_indices.numel() >= indices.numel()
    _check("dmt_sptt_peer_permute_ids", _lib.dmt_sptt_peer_permute_ids(
        _ptr(indices), _ptr(offsets), features, G, L, B_l, indices.numel(), _ptr(out_indices),
        _ptr(out_offsets), _stream(stream)))


def dmt_plan_set_row_shards(plan: dmt_plan, row_begin: Sequence[int]) -> None:
    assert len(row_begin) == plan.num_tables
    arr = (ctypes.c_int64 * plan.num_tables)(*[int(r) for r in row_begin])
    _check("dmt_plan_set_row_shards", _lib.dmt_plan_set_row_shards(plan.handle, arr))
