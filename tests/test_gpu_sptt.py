"""GPU parity of SPTT's shuffle steps (dmt_sptt_peer_permute, dmt_sptt_shuffle) against the
oracle: pure data movement, so every comparison is bit for bit."""
import numpy as np
import pytest
import torch

import paper_2403_00877_amd as dmt
from oracle import sptt

pytestmark = pytest.mark.gpu


def _blocks(rng, shape, dtype):
    """Random bit patterns of the given element type (any bits: the kernels only move them)."""
    nbytes = int(np.prod(shape)) * np.dtype(dtype).itemsize
    return rng.integers(0, 256, size=nbytes, dtype=np.uint8).view(dtype).reshape(shape)


@pytest.mark.parametrize("F,G,L,Bl,N,dtype", [
    (1, 4, 2, 3, 8, np.uint16),        # the paper's example: 4 GPUs, 2 per host, one feature each
    (8, 8, 4, 129, 128, np.uint16),    # Mid's feature shape on one 8-GPU tower split 2 hosts x 4
    (3, 16, 8, 5, 32, np.float32),
    (5, 6, 3, 1, 4, np.float32),       # one 16-byte unit per block
    (2, 8, 1, 7, 8, np.uint16),        # one GPU per host: peer order = rank order
    (2, 8, 8, 7, 8, np.uint16),        # one host: peer order = rank order as well
    (1, 2, 2, 4097, 128, np.uint16),   # blocks longer than one workgroup pass, ragged tail
    (64, 8, 4, 1024, 128, np.uint16),  # the size bench.py times: Mid's pooled tensor, 134 MB
])
def test_peer_permute_matches_the_oracle(F, G, L, Bl, N, dtype):
    rng = np.random.default_rng(F * 100 + G)
    x = _blocks(rng, (F, G, Bl, N), dtype)
    block_bytes = Bl * N * x.itemsize
    d_in = torch.from_numpy(x.view(np.uint8).reshape(-1)).cuda()
    d_out = torch.zeros_like(d_in)
    dmt.dmt_sptt_peer_permute(d_in, d_out, F, G, L, block_bytes)
    torch.cuda.synchronize()
    got = d_out.cpu().numpy().view(dtype).reshape(F, G, Bl, N)
    np.testing.assert_array_equal(got, sptt.peer_permute(x, L))
    assert dmt.dmt_sptt_peer_order(G, L) == sptt.peer_order(G, L)


@pytest.mark.parametrize("F,P,Bl,N,dtype", [(1, 1, 2, 8, np.uint16), (8, 2, 129, 128, np.uint16),
                                            (16, 16, 33, 64, np.uint16), (3, 5, 1, 4, np.float32),
                                            (2, 3, 2049, 128, np.float32),
                                            (64, 8, 1024, 128, np.uint16)])      # 134 MB, as bench.py times it
def test_shuffle_matches_the_oracle(F, P, Bl, N, dtype):
    rng = np.random.default_rng(F * 100 + P)
    z = _blocks(rng, (F, P, Bl, N), dtype)
    block_bytes = Bl * N * z.itemsize
    d_in = torch.from_numpy(z.view(np.uint8).reshape(-1)).cuda()
    d_out = torch.zeros_like(d_in)
    dmt.dmt_sptt_shuffle(d_in, d_out, F, P, block_bytes)
    torch.cuda.synchronize()
    got = d_out.cpu().numpy().view(dtype).reshape(P, F, Bl, N)
    np.testing.assert_array_equal(got, sptt.shuffle(z))


@pytest.mark.parametrize("T,L,per_tower", [(2, 2, [1, 1]), (2, 4, [5, 4]), (3, 2, [2, 3, 1])])
def test_the_six_steps_with_the_device_kernels_keep_the_lookup(T, L, per_tower):
    """A simulated cluster: steps c and e of every virtual GPU run on the device, the exchanges
    (d, f) are host copies; every GPU must end up with the plain lookup's embeddings of all
    towers' features for its own samples."""
    rng = np.random.default_rng(7)
    B_l, N = 5, 8
    G = T * L
    tower_tables, k = [], 0
    for n in per_tower:
        tower_tables.append(list(range(k, k + n)))
        k += n
    F = k
    truth = rng.normal(size=(F, G * B_l, N)).astype(np.float32)
    block_bytes = B_l * N * 4

    def on_device(fn, x, *dims):
        d_in = torch.from_numpy(np.ascontiguousarray(x).view(np.uint8).reshape(-1)).cuda()
        d_out = torch.zeros_like(d_in)
        fn(d_in, d_out, *dims, block_bytes)
        torch.cuda.synchronize()
        return d_out.cpu().numpy().view(np.float32)

    local = [[f for i, f in enumerate(fs) if i % L == l] for fs in tower_tables for l in range(L)]
    permuted = []
    for r in range(G):
        if not local[r]:
            permuted.append(None)
            continue
        held = np.stack([truth[f].reshape(G, B_l, N) for f in local[r]])           # steps a + b
        permuted.append(on_device(dmt.dmt_sptt_peer_permute, held, len(local[r]), G, L)
                        .reshape(len(local[r]), G, B_l, N))                          # step c
    shuffled = []
    for r in range(G):
        t, l = divmod(r, L)
        parts, names = [], []
        for src in range(t * L, (t + 1) * L):                                       # step d
            if permuted[src] is not None:
                parts.append(permuted[src][:, l * T:(l + 1) * T])
                names += local[src]
        z = np.concatenate(parts, axis=0)[np.argsort([tower_tables[t].index(f) for f in names])]
        shuffled.append(on_device(dmt.dmt_sptt_shuffle, z, len(names), T)
                        .reshape(T, len(names), B_l, N))                             # step e
    ref = sptt.simulate(lambda f, lo, hi: truth[f, lo:hi], tower_tables, L, B_l)
    for r in range(G):
        t, l = divmod(r, L)
        for src_host in range(T):                                                   # step f
            got = shuffled[src_host * L + l][t]
            np.testing.assert_array_equal(got, ref[r][src_host])
            for i, f in enumerate(tower_tables[src_host]):
                np.testing.assert_array_equal(got[i], truth[f, r * B_l:(r + 1) * B_l])


def test_shuffle_steps_reject_bad_arguments():
    raw_p = dmt.binding._lib.dmt_sptt_peer_permute
    raw_s = dmt.binding._lib.dmt_sptt_shuffle
    a = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    b = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    pa, pb = a.data_ptr(), b.data_ptr()
    assert raw_p(pa, pb, 2, 4, 2, 64, None) == 0
    assert raw_p(None, pb, 2, 4, 2, 64, None) == 1 and raw_p(pa, None, 2, 4, 2, 64, None) == 1
    assert raw_p(pa, pa, 2, 4, 2, 64, None) == 1              # in place
    assert raw_p(pa, pb, 2, 4, 3, 64, None) == 1              # L does not divide G
    assert raw_p(pa, pb, 2, 4, 2, 24, None) == 1              # block not a multiple of 16 bytes
    assert raw_p(pa + 4, pb, 2, 4, 2, 64, None) == 1          # misaligned
    assert raw_p(pa, pb, 0, 4, 2, 64, None) == 1
    assert raw_s(pa, pb, 2, 4, 64, None) == 0
    assert raw_s(pa, pb, 2, 0, 64, None) == 1 and raw_s(pa, pb, 2, 4, 0, None) == 1
    assert raw_s(pa, pb, 1 << 21, 4, 64, None) == 2           # beyond the supported block count
    torch.cuda.synchronize()


def _jagged(rng, nbags, max_len, rows, empty=0.2):
    lens = rng.integers(0, max_len + 1, size=nbags)
    lens[rng.random(nbags) < empty] = 0
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    return rng.integers(0, rows, size=int(off[-1])).astype(np.int32), off


@pytest.mark.parametrize("F,G,L,Bl,max_len", [
    (1, 4, 2, 1, 3),          # the paper's example: 4 GPUs, 2 per host
    (3, 8, 4, 5, 7), (2, 6, 3, 33, 40), (5, 8, 1, 4, 2), (5, 8, 8, 4, 2),
    (8, 8, 4, 1024, 40),      # Mid's feature shape: 8192 samples over 8 ranks, ~20 ids per bag
    (2, 16, 4, 300, 900),     # blocks of ids that span many workgroup passes
    (4, 4, 2, 6, 0),          # no ids at all
])
def test_peer_permute_of_the_sparse_inputs_matches_the_oracle(F, G, L, Bl, max_len):
    """Steps b and c swapped (Sec. 3.1.3): the permute on ids, bit for bit."""
    rng = np.random.default_rng(F * 1000 + G * 10 + L)
    idx, off = _jagged(rng, F * G * Bl, max_len, 1 << 20)
    d_idx, d_off = torch.from_numpy(idx).cuda(), torch.from_numpy(off).cuda()
    o_idx = torch.full((max(len(idx), 1),), -7, dtype=torch.int32, device="cuda")
    o_off = torch.full((len(off),), -7, dtype=torch.int64, device="cuda")
    dmt.dmt_sptt_peer_permute_ids(d_idx, d_off, F, G, L, Bl, o_idx[:len(idx)], o_off)
    torch.cuda.synchronize()
    want_idx, want_off = sptt.peer_permute_ids(idx, off, F, G, L, Bl)
    np.testing.assert_array_equal(o_off.cpu().numpy(), want_off)
    np.testing.assert_array_equal(o_idx[:len(idx)].cpu().numpy(), want_idx)


def test_lookup_on_permuted_ids_is_the_permuted_lookup_on_the_device():
    """b and c swapped against b then c, both on the device: same bits."""
    import workloads as wl
    from harness import DeviceWorkload
    G, L = 8, 4
    w = wl.scaled(wl.mid(), max_rows=5000, batch=G * 37, num_tables=8)
    w.pooled_dtype = "f32"
    w.table_to_tower = [0] * 8
    w.tm_out = [256]
    dw = DeviceWorkload(w)
    F, B, N = 8, w.batch, 128
    Bl = B // G
    idx, off = wl.lookup_batch(w)
    d_idx, d_off = torch.from_numpy(idx).cuda(), torch.from_numpy(off).cuda()
    p_idx, p_off = torch.empty_like(d_idx), torch.empty_like(d_off)
    dmt.dmt_sptt_peer_permute_ids(d_idx, d_off, F, G, L, Bl, p_idx, p_off)
    torch.cuda.synchronize()
    swapped = dw.lookup(p_idx.cpu().numpy(), p_off.cpu().numpy())        # [B][F][N], samples in peer order
    plain = dw.lookup(idx, off)
    # step c on the plain lookup, per feature: (F, G, Bl * N) blocks
    blocks = plain.view(B, F, N).permute(1, 0, 2).contiguous().view(-1)
    out = torch.empty_like(blocks)
    dmt.dmt_sptt_peer_permute(blocks.view(torch.uint8), out.view(torch.uint8), F, G, L, Bl * N * 4)
    torch.cuda.synchronize()
    want = out.view(F, B, N).permute(1, 0, 2).contiguous().view(-1)
    assert torch.equal(swapped.view(torch.int32), want.view(torch.int32))


def test_peer_permute_of_ids_rejects_bad_arguments():
    raw = dmt.binding._lib.dmt_sptt_peer_permute_ids
    i = torch.zeros(64, dtype=torch.int32, device="cuda")
    o = torch.zeros(4 * 2 + 1, dtype=torch.int64, device="cuda")
    i2, o2 = torch.zeros_like(i), torch.zeros_like(o)
    a = (i.data_ptr(), o.data_ptr())
    assert raw(*a, 1, 4, 2, 2, 0, i2.data_ptr(), o2.data_ptr(), None) == 0
    assert raw(*a, 1, 4, 3, 2, 0, i2.data_ptr(), o2.data_ptr(), None) == 1       # L does not divide G
    assert raw(*a, 1, 4, 2, 2, 0, i2.data_ptr(), o.data_ptr(), None) == 1        # offsets in place
    assert raw(*a, 1, 4, 2, 2, 8, i.data_ptr(), o2.data_ptr(), None) == 1        # ids in place
    assert raw(None, o.data_ptr(), 1, 4, 2, 2, 8, i2.data_ptr(), o2.data_ptr(), None) == 1
    assert raw(*a, 1, 2048, 2, 2, 0, i2.data_ptr(), o2.data_ptr(), None) == 2    # more ranks than supported
    torch.cuda.synchronize()


@pytest.mark.parametrize("seed", range(24))
def test_random_shapes_of_all_three_shuffles(seed):
    """Seeded arbitrary feature / rank / block counts through the block permute (step c), the
    block transpose (step e) and the permute on ids (steps b and c swapped), bit for bit."""
    rng = np.random.default_rng([91, seed])
    F = int(rng.integers(1, 20))
    L = int(rng.choice([1, 2, 3, 4, 8]))
    G = L * int(rng.integers(1, 9))
    Bl = int(np.exp(rng.uniform(0, np.log(600))))
    N = int(rng.choice([4, 8, 16, 32, 128]))
    z = rng.integers(0, 2**31, size=(F, G, Bl, N), dtype=np.int64).astype(np.uint32)
    d_in = torch.from_numpy(z.view(np.uint8).reshape(-1)).cuda()
    d_out = torch.zeros_like(d_in)
    dmt.dmt_sptt_peer_permute(d_in, d_out, F, G, L, Bl * N * 4)
    torch.cuda.synchronize()
    order = sptt.peer_order(G, L)
    np.testing.assert_array_equal(d_out.cpu().numpy().view(np.uint32).reshape(F, G, Bl, N), z[:, order])
    d_out.zero_()
    dmt.dmt_sptt_shuffle(d_in, d_out, F, G, Bl * N * 4)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(d_out.cpu().numpy().view(np.uint32).reshape(G, F, Bl, N),
                                  z.transpose(1, 0, 2, 3))
    idx, off = _jagged(rng, F * G * Bl, int(rng.choice([0, 2, 9, 60])), 1 << 20, empty=float(rng.random()) * 0.8)
    d_idx, d_off = torch.from_numpy(idx).cuda(), torch.from_numpy(off).cuda()
    o_idx = torch.full((max(len(idx), 1),), -7, dtype=torch.int32, device="cuda")
    o_off = torch.full((len(off),), -7, dtype=torch.int64, device="cuda")
    dmt.dmt_sptt_peer_permute_ids(d_idx, d_off, F, G, L, Bl, o_idx[:len(idx)], o_off)
    torch.cuda.synchronize()
    want_idx, want_off = sptt.peer_permute_ids(idx, off, F, G, L, Bl)
    np.testing.assert_array_equal(o_off.cpu().numpy(), want_off)
    np.testing.assert_array_equal(o_idx[:len(idx)].cpu().numpy(), want_idx)
