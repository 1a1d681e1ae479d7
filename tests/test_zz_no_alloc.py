"""dmt_tower_lookup_bwd_update_noalloc (scratch inside the library) against
dmt_tower_lookup_bwd_update (caller's workspace): same kernels, so tables and states must
come out bit for bit alike; two calls in a row, the second on a smaller batch of lookups."""
import numpy as np
import pytest
import torch

import workloads as wl
from harness import DeviceWorkload

pytestmark = pytest.mark.gpu


def _inputs(w, batch_id, keep_bags=None):
    idx, off = wl.lookup_batch(w, batch_id)
    grad = wl.grad_pooled(w, batch_id)
    if keep_bags is not None:            # a smaller input: only every keep_bags-th bag keeps its ids
        lens = np.diff(off)
        keep = (np.arange(len(lens)) % keep_bags) == 0
        mask = np.repeat(keep, lens)
        idx = np.ascontiguousarray(idx[mask])
        off = np.concatenate([[0], np.cumsum(np.where(keep, lens, 0))]).astype(np.int64)
    return idx, off, grad


def _bits(t):
    return t.view(torch.int16 if t.element_size() == 2 else torch.int32)


@pytest.mark.parametrize("name", ["tiny", "mid"])
def test_noalloc_matches_the_workspace_entry_point(name):
    w = wl.tiny() if name == "tiny" else wl.scaled(wl.mid(), max_rows=5000, batch=256, num_tables=16)
    ref = DeviceWorkload(w, with_state=True)
    new = DeviceWorkload(w, with_state=True)
    dmt = ref.dmt
    assert dmt.dmt_bwd_noalloc_scratch_bytes() == 32 << 20
    for call, keep_bags in enumerate([None, 3]):
        idx, off, grad = _inputs(w, call, keep_bags)
        d_idx, d_off = torch.from_numpy(idx).cuda(), torch.from_numpy(off).cuda()
        d_grad = torch.from_numpy(grad).cuda()
        nbytes = dmt.dmt_bwd_workspace_bytes(ref.plan, w.batch, len(idx))
        assert nbytes <= dmt.dmt_bwd_noalloc_scratch_bytes()
        ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        dmt.dmt_tower_lookup_bwd_update(ref.plan, d_idx, d_off, w.batch, d_grad, w.lr, w.eps, ws)
        dmt.dmt_tower_lookup_bwd_update_noalloc(new.plan, d_idx, d_off, w.batch, d_grad, w.lr, w.eps)
        torch.cuda.synchronize()
        assert dmt.dmt_last_device_error(ref.plan) == -1
        assert dmt.dmt_last_device_error(new.plan) == -1
        touched = 0
        for f in range(w.num_tables):
            assert torch.equal(_bits(ref.tables[f]), _bits(new.tables[f])), (call, f)
            assert torch.equal(ref.states[f], new.states[f]), (call, f)
            touched += int((new.states[f] != 0).sum())
        assert touched > 0


def test_noalloc_rejects_what_does_not_fit():
    w = wl.tiny()
    dw = DeviceWorkload(w, with_state=True, max_nnz=1 << 26)
    dmt = dw.dmt
    nnz = 1 << 25                                   # far beyond the array: must fail before any launch
    assert dmt.dmt_bwd_workspace_bytes(dw.plan, w.batch, nnz) > dmt.dmt_bwd_noalloc_scratch_bytes()
    idx = torch.zeros(nnz, dtype=torch.int32, device="cuda")
    off = torch.zeros(w.num_tables * w.batch + 1, dtype=torch.int64, device="cuda")
    grad = torch.zeros(dw.base[-1], dtype=torch.float32, device="cuda")
    with pytest.raises(dmt.DmtError) as e:
        dmt.dmt_tower_lookup_bwd_update_noalloc(dw.plan, idx, off, w.batch, grad, w.lr, w.eps)
    assert e.value.code == 4                        # DMT_ENOMEM


@pytest.mark.parametrize("seed", range(12))
def test_noalloc_on_random_configurations(seed):
    """Arbitrary table sets: the scratch-array entry point and the workspace one leave the same
    bits, whichever segment-reduce kernel the widths select."""
    from test_gpu_random_shapes import random_workload
    w = random_workload(900 + seed)
    ref = DeviceWorkload(w, with_state=True)
    new = DeviceWorkload(w, with_state=True)
    dmt = ref.dmt
    idx, off, grad = _inputs(w, 0)
    nbytes = dmt.dmt_bwd_workspace_bytes(ref.plan, w.batch, len(idx))
    if nbytes > dmt.dmt_bwd_noalloc_scratch_bytes():
        pytest.skip("does not fit the scratch array")
    d_idx, d_off = torch.from_numpy(idx).cuda(), torch.from_numpy(off).cuda()
    d_grad = torch.from_numpy(grad).cuda()
    ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
    dmt.dmt_tower_lookup_bwd_update(ref.plan, d_idx, d_off, w.batch, d_grad, w.lr, w.eps, ws)
    dmt.dmt_tower_lookup_bwd_update_noalloc(new.plan, d_idx, d_off, w.batch, d_grad, w.lr, w.eps)
    torch.cuda.synchronize()
    assert dmt.dmt_last_device_error(ref.plan) == -1 and dmt.dmt_last_device_error(new.plan) == -1
    for f in range(w.num_tables):
        assert torch.equal(_bits(ref.tables[f]), _bits(new.tables[f])), f
        assert torch.equal(ref.states[f], new.states[f]), f
