"""The two calibration kernels (a copy and a row gather of known traffic) do what their
declarations say: the measurements built on them mean nothing otherwise."""
import numpy as np
import pytest
import torch

import paper_2403_00877_amd as dmt

pytestmark = pytest.mark.gpu


def test_calibration_copy_copies():
    src = torch.arange(1 << 20, dtype=torch.int32, device="cuda")
    dst = torch.zeros_like(src)
    dmt.dmt_calibration_copy(dst, src)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)


@pytest.mark.parametrize("row_bytes,rows,n", [(256, 1000, 70001), (64, 37, 5000), (16, 5, 129), (1024, 64, 3000)])
def test_calibration_gather_reads_every_row_it_is_given(row_bytes, rows, n):
    """Each thread's folded word is the exclusive-or of the 16-byte chunks the kernel's own
    assignment gives it: row i of the list goes to wave (i / (rows per step)) % waves, its
    chunks to the lanes of sub-group i % rows-per-instruction."""
    rng = np.random.default_rng(row_bytes + n)
    table = rng.integers(0, 2**32, size=(rows, row_bytes // 4), dtype=np.uint32)
    ids = rng.integers(0, rows, size=n).astype(np.int32)
    ids[::97] = rows + 5                      # outside the table: row 0 is read instead
    ids[1::101] = -3
    blocks = dmt.binding.DMT_CALIBRATION_GATHER_BLOCKS
    d_out = torch.zeros(blocks * 256 * 4, dtype=torch.int32, device="cuda")
    dmt.dmt_calibration_gather(torch.from_numpy(table.view(np.int32)).cuda(), row_bytes,
                               torch.from_numpy(ids).cuda(), d_out)
    torch.cuda.synchronize()
    got = d_out.cpu().numpy().view(np.uint32).reshape(blocks * 256, 4)

    lpr = row_bytes // 16
    rpi = 64 // lpr
    per_step = rpi * 8
    nwaves = blocks * 256 // 64
    i = np.arange(n)
    wave = (i // per_step) % nwaves
    sub = (i % per_step) % rpi
    r = np.where((ids >= 0) & (ids < rows), ids, 0)
    want = np.zeros((blocks * 256, 4), dtype=np.uint32)
    chunks = table.reshape(rows, lpr, 4)
    for c in range(lpr):
        np.bitwise_xor.at(want, wave * 64 + sub * lpr + c, chunks[r, c])
    assert np.array_equal(got, want)


def test_calibration_gather_rejects_bad_arguments():
    t = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    ids = torch.zeros(8, dtype=torch.int32, device="cuda")
    out = torch.zeros(dmt.binding.DMT_CALIBRATION_GATHER_BLOCKS * 256 * 16, dtype=torch.uint8, device="cuda")
    for bad in (24, 8, 2048):
        with pytest.raises(dmt.DmtError):
            dmt.dmt_calibration_gather(t, bad, ids, out)
