"""GPU checks of the input generator's device helpers against their numpy forms:
the block regenerator and the position-sensitive block hash that the full-size
parity tests rest on."""
import numpy as np
import pytest
import torch

import kvm_workload as wl
from kvm_workload import device as wl_device

from gpu_util import DEV

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("m", [wl.TINY, wl.Model("gqa", 2, 8, 32, 128, 16, "bf16")], ids=["tiny_f16", "gqa_bf16"])
def test_device_fill_and_block_regenerator_equal_the_host_generator(m):
    n_blocks, seed = 40, 77
    mem = torch.empty(n_blocks * m.block_bytes, dtype=torch.uint8, device=DEV)
    wl_device.fill_pool(mem, m, n_blocks, seed, wl.STREAM_DST)
    host = wl.gen_pool_host(seed, wl.STREAM_DST, m, n_blocks)
    assert np.array_equal(mem.cpu().numpy().view(np.uint16), host)
    ids = np.array([39, 0, 7, 7, 65535, 123456, 2**31 - 1], dtype=np.int32)
    run = m.H * m.B * m.D
    out = torch.zeros(len(ids) * run + 64, dtype=torch.int16, device=DEV)
    for plane in (0, 2 * m.L - 1):
        wl_device.gen_blocks(out, torch.from_numpy(ids).to(DEV), m, seed, wl.STREAM_SRC, plane)
        got = out.cpu().numpy().view(np.uint16)
        assert (got[len(ids) * run:] == 0).all()                       # nothing past the last block
        exp = wl.gen_blocks(seed, wl.STREAM_SRC, m, plane, ids.astype(np.int64))
        assert np.array_equal(got[:len(ids) * run].reshape(exp.shape), exp)
        for i, b in enumerate(ids):                                       # and the one-block form
            assert np.array_equal(exp[i], wl.gen_block(seed, wl.STREAM_SRC, m, plane, int(b)))


def test_block_hash_matches_numpy_and_sees_moved_words():
    m = wl.TINY
    n_blocks, seed = 24, 78
    mem = torch.empty(n_blocks * m.block_bytes, dtype=torch.uint8, device=DEV)
    wl_device.fill_pool(mem, m, n_blocks, seed, wl.STREAM_SRC)
    host = mem.cpu().numpy().view(np.uint16).reshape(2 * m.L, n_blocks, -1)
    h = wl_device.plane_block_hashes(mem, m, n_blocks).cpu().numpy().view(np.uint64)
    for p in range(2 * m.L):
        for b in range(n_blocks):
            assert int(h[p, b]) == wl_device.block_hash_host(host[p, b])
    # swap two 16-byte vectors inside (plane 1, block 5): a plain sum of the words is
    # unchanged, the hash is not; no other block's hash moves
    v = mem.view(torch.int64).view(2 * m.L, n_blocks, -1)
    plain_before = int(v[1, 5].sum())
    a, b = v[1, 5, 0:2].clone(), v[1, 5, 10:12].clone()
    assert not torch.equal(a, b)
    v[1, 5, 0:2], v[1, 5, 10:12] = b, a
    assert int(v[1, 5].sum()) == plain_before
    h2 = wl_device.plane_block_hashes(mem, m, n_blocks).cpu().numpy().view(np.uint64)
    diff = h2 != h
    assert diff[1, 5] and diff.sum() == 1
