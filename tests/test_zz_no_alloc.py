"""GPU test of kvm_paged_decode_static, the entry point for callers that cannot
allocate device memory: its context-split workspace is the library's static
device array instead of a caller buffer.

Called through the C ABI on two batches in a row, the second smaller than the
first (so the second call finds the first call's leftovers in the array); each
result must equal kvm_paged_decode's with a caller workspace bit for bit (same
kernels, same split plan) and lie within 2e-3 of the fp64 oracle.  Between and
around the calls no torch allocation is made on the device.
"""
import numpy as np
import pytest
import torch

import kvm_workload as wl
import paper_2501_06709_amd as kvm

from gpu_util import DEV, Side, make_pair, to_dev

pytestmark = pytest.mark.gpu
TOL = 2e-3


def case(m, lens, seed, n_blocks):
    src, _ = make_pair(m, n_blocks, 8, lens, [0] * len(lens), seed=seed, finite=True)
    side = Side(m, n_blocks, src.host, src.tables, lens)
    q = wl.gen_q(seed, m, len(lens))
    return side, q


@pytest.mark.parametrize("m", [wl.Model("gqa4", 2, 2, 8, 128, 16, "bf16"),
                               wl.Model("mha64", 2, 4, 4, 64, 16, "f16")], ids=["gqa4_bf16", "mha64_f16"])
def test_static_scratch_decode_equals_workspace_decode_twice(oracle, m):
    # first batch: long contexts, split 16 ways; second: fewer, shorter requests,
    # split 2 to 4 ways, run straight after it on the same stream
    big, q_big = case(m, [4096, 3000, 1111], 61, 600)
    small, q_small = case(m, [700, 90], 62, 64)
    sides = [(big, q_big), (small, q_small)]
    need = [kvm.kvm_decode_workspace_bytes(s.layout, s.batch) for s, _ in sides]
    assert need[0] > need[1] > 0, need           # both calls really use the scratch
    assert need[0] <= kvm.KVM_STATIC_SCRATCH_BYTES
    # everything the calls touch is allocated before the first of them
    q_dev = [to_dev(q) for _, q in sides]
    out_ws = [torch.full(q.shape, 7.0, dtype=torch.float32, device=DEV) for _, q in sides]
    out_st = [torch.full(q.shape, 9.0, dtype=torch.float32, device=DEV) for _, q in sides]
    ws = [torch.empty(n, dtype=torch.uint8, device=DEV) for n in need]
    for i, (s, _) in enumerate(sides):
        kvm.kvm_paged_decode(s.pool, s.batch, q_dev[i], out_ws[i], workspace=ws[i])
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for i, (s, _) in enumerate(sides):           # two calls in a row, no sync between them
        kvm.kvm_paged_decode_static(s.pool, s.batch, q_dev[i], out_st[i])
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    for i, (s, q) in enumerate(sides):
        assert torch.equal(out_st[i], out_ws[i]), "call %d differs from kvm_paged_decode" % i
        ref = oracle.paged_decode(s.host, s.st, m.L, m.H, m.Hq, m.D, m.B, m.dtype, s.off, s.blk, s.k, q)
        err = np.abs(out_st[i].cpu().numpy() - ref).max()
        assert err < TOL, (i, err)


def test_static_scratch_16bit_output_and_unsplit_batch(oracle):
    """A batch that needs no split runs without touching the array; a 16-bit output
    goes through the same path."""
    m = wl.Model("gqa4", 2, 2, 8, 128, 16, "bf16")
    side, q = case(m, [40, 17, 333] * 30, 63, 1024)      # 90 requests: more than one launch, no split
    assert kvm.kvm_decode_workspace_bytes(side.layout, side.batch) == 0
    q_dev = to_dev(q)
    a = torch.zeros(q.shape, dtype=torch.int16, device=DEV)
    b = torch.zeros(q.shape, dtype=torch.int16, device=DEV)
    kvm.kvm_paged_decode(side.pool, side.batch, q_dev, a, out_is_f32=False)
    kvm.kvm_paged_decode_static(side.pool, side.batch, q_dev, b, out_is_f32=False)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    long_side, q2 = case(m, [2048], 64, 256)
    q2_dev = to_dev(q2)
    a = torch.zeros(q2.shape, dtype=torch.int16, device=DEV)
    b = torch.zeros(q2.shape, dtype=torch.int16, device=DEV)
    ws = torch.empty(kvm.kvm_decode_workspace_bytes(long_side.layout, long_side.batch), dtype=torch.uint8,
                     device=DEV)
    kvm.kvm_paged_decode(long_side.pool, long_side.batch, q2_dev, a, out_is_f32=False, workspace=ws)
    kvm.kvm_paged_decode_static(long_side.pool, long_side.batch, q2_dev, b, out_is_f32=False)
    torch.cuda.synchronize()
    assert torch.equal(a, b)
    ref = oracle.paged_decode(long_side.host, long_side.st, m.L, m.H, m.Hq, m.D, m.B, m.dtype,
                              long_side.off, long_side.blk, long_side.k, q2)
    got = wl.bits16_to_f64(b.cpu().numpy().view(np.uint16), m.dtype)
    assert np.abs(got - ref).max() < 2 ** -7     # one bf16 unit in the last place below 2


def test_static_scratch_holds_a_forced_64_way_split():
    m = wl.Model("gqa4", 8, 2, 8, 128, 16, "bf16")
    lens = [16384] * 4
    lay = kvm.kvm_layout_canonical(m.L, m.H, m.Hq, m.D, m.B, m.dtype, 4096)
    tabs = [np.arange(r * 1024, (r + 1) * 1024, dtype=np.int32) for r in range(4)]
    off = np.arange(5, dtype=np.int32) * 1024
    blk = np.concatenate(tabs)
    pool_mem = torch.zeros(kvm.kvm_pool_span_bytes(lay, 4096), dtype=torch.uint8, device=DEV)
    pool = kvm.Pool(pool_mem, 4096, lay)
    batch = kvm.Batch(off, blk, lens, torch.from_numpy(blk).to(DEV))
    q = torch.zeros((4, m.L, m.Hq, m.D), dtype=torch.int16, device=DEV)
    out = torch.full(q.shape, 5.0, dtype=torch.float32, device=DEV)
    try:
        kvm.kvm_set_option("decode.force_splits", 64)   # 4*8*8*64*130*4 = 8.5 MB: fits
        assert kvm.kvm_decode_workspace_bytes(lay, batch) <= kvm.KVM_STATIC_SCRATCH_BYTES
        kvm.kvm_paged_decode_static(pool, batch, q, out)
        torch.cuda.synchronize()
        assert not (out == 5.0).any()
    finally:
        kvm.kvm_set_option("reset", 0)
