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


def test_reference_copy_moves_the_chunks_it_says():
    """The table-free reference kernel the benchmark times (runs at consecutive or permuted
    slots, chunks of a run optionally shifted by some dies) is a copy: every chunk of the
    source arrives exactly once, where the host's model of the kernel puts it."""
    run, n_runs, slots = 32768, 48, 64
    rng = np.random.default_rng(5)
    src_h = rng.integers(0, 2**31, size=slots * run // 4, dtype=np.int32)
    src = torch.from_numpy(src_h).to(DEV)
    sink = torch.zeros(4, dtype=torch.int32, device=DEV)

    def perm(r, bits, key):
        if bits == 0:
            return r
        mask, h = (1 << bits) - 1, (bits + 1) // 2
        r = (r + key) & mask
        r = (r * 0x9E3779B97F4A7C15) & mask
        r ^= r >> h
        r = ((r << h) | (r >> (bits - h))) & mask
        r = (r * 0xBF58476D1CE4E5B9) & mask
        r ^= r >> h
        r = (r * 0x94D049BB133111EB) & mask
        r ^= r >> h
        return r

    key_s, key_d = 0, 0x5851F42D4C957F2D
    for s_rand, d_rand, s_rot, d_rot in ((False, False, 0, 0), (True, False, 1, 0), (False, True, 0, 3), (True, True, 5, 2),
                                         (False, False, 8, 0), (True, True, 9, 8)):
        dst = torch.full_like(src, -1)
        wl_device.ref_stream(wl_device.REF_COPY, src, dst, run, n_runs, s_rand, d_rand, sink, s_rot, d_rot)
        torch.cuda.synchronize()
        exp = np.full_like(src_h, -1).reshape(slots, 8, 1024)
        s3 = src_h.reshape(slots, 8, 1024)
        for r in range(n_runs):
            for c in range(8):
                exp[perm(r, 6 if d_rand else 0, key_d), (c + (d_rot & 7) + (d_rot >> 3) * (r % 8)) % 8] = \
                    s3[perm(r, 6 if s_rand else 0, key_s), (c + (s_rot & 7) + (s_rot >> 3) * (r % 8)) % 8]
        assert np.array_equal(dst.cpu().numpy().reshape(slots, 8, 1024), exp), (s_rand, d_rand, s_rot, d_rot)


def test_reference_walk_runs_in_bounds_sizes():
    """The walking read kernel only reads: it must accept the sizes the benchmark uses and
    refuse a stride that would leave the buffer."""
    buf = torch.zeros(64 << 20, dtype=torch.uint8, device=DEV)           # 2 x 8192 pieces
    sink = torch.zeros(4, dtype=torch.int32, device=DEV)
    for stride, sliced in ((1, True), (256, True), (256, False), (2000, True)):
        assert wl_device.ref_walk(buf, 16 << 20, stride, 16, sliced, sink) == 16 << 20
    torch.cuda.synchronize()
    with pytest.raises(AssertionError):
        wl_device.ref_walk(buf, 16 << 20, 3000, 16, True, sink)                  # 3 * 3000 >= 8192 pieces
    assert int(sink.sum()) == 0
