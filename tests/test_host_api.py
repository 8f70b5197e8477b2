"""CPU-side checks of libkvm: it loads without a GPU, exports every symbol the
header declares, computes the closed-form sizes, rejects bad arguments before
any launch, and its free list behaves like the oracle's (itself pinned by brute
force).  No kernel is launched here: every call below either is pure host code
or fails validation first.
"""
import ctypes
import os
import re

import numpy as np
import pytest

import kvm_workload as wl
import paper_2501_06709_amd as kvm
from paper_2501_06709_amd import build as kvm_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000000000  # stands in for a device address; validation never dereferences it


@pytest.fixture(scope="module", autouse=True)
def built():
    if kvm_build.stale():
        kvm_build.build()
    kvm.lib()


def test_every_declared_symbol_is_exported():
    text = open(os.path.join(ROOT, "include", "kvm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(kvm_[a-z_0-9]+)\s*\(", text))
    assert {"kvm_pack", "kvm_unpack", "kvm_migrate", "kvm_paged_decode", "kvm_freelist_alloc",
            "kvm_bytes_per_token", "kvm_staging_bytes"} <= names
    L = ctypes.CDLL(kvm.binding.LIB_PATH)
    for n in sorted(names):
        assert hasattr(L, n), n


def test_sizes_closed_form_and_paper_value():
    lay = kvm.kvm_layout_canonical(40, 40, 40, 128, 16, "f16", 64)
    assert kvm.kvm_bytes_per_token(lay) == 819200          # 13B: 40*2*40*128*2
    assert kvm.kvm_bytes_per_token(lay) * 4096 == 3355443200  # "about 3.2 GB" per 4096-token request
    assert kvm.kvm_block_bytes(lay) == 16 * 819200
    assert kvm.kvm_pool_span_bytes(lay, 64) == 64 * 16 * 819200
    for m in (wl.TINY, wl.LLAMA2_7B, wl.LLAMA3_8B, wl.LLAMA2_13B):
        lay = kvm.kvm_layout_canonical(m.L, m.H, m.Hq, m.D, m.B, m.dtype, 8)
        assert kvm.kvm_bytes_per_token(lay) == m.bytes_per_token
        st = wl.canonical_strides(m, 8)
        assert [lay.stride_layer, lay.stride_kv, lay.stride_block, lay.stride_head,
                lay.stride_slot] == list(st)
        b = kvm.Batch([0, 2, 2, 5], [0, 1, 2, 3, 4], [17, 0, 48], FAKE)
        assert kvm.kvm_staging_bytes(lay, b) == 65 * m.bytes_per_token


def test_layout_validation():
    for args in ((0, 4, 4, 64, 16, "f16", 8), (2, 4, 6, 64, 16, "f16", 8), (2, 4, 4, 60, 16, "f16", 8),
                 (2, 4, 4, 64, 16, 5, 8), (2, 4, 4, 64, 16, "f16", 0)):
        with pytest.raises(kvm.KvmError) as e:
            kvm.kvm_layout_canonical(*args)
        assert e.value.status == kvm.KVM_EINVAL
    lay = kvm.kvm_layout_canonical(2, 4, 4, 64, 16, "f16", 8)
    lay.stride_slot = 60
    assert kvm.kvm_bytes_per_token(lay) == -1 and kvm.kvm_pool_span_bytes(lay, 8) == -1
    # a block whose head and slot strides span more than 2^32 bytes is refused
    # (the kernels keep a lane's offset inside one block in 32 bits)
    lay = kvm.kvm_layout_canonical(2, 4, 4, 64, 16, "f16", 8)
    lay.stride_head = 1 << 30
    assert kvm.kvm_bytes_per_token(lay) == -1
    lay.stride_head = (1 << 29)            # 3 * 2^29 + ... elements: still below 2^31
    assert kvm.kvm_bytes_per_token(lay) == 2 * 2 * 4 * 64 * 2


def _pool(n_blocks=32, m=wl.TINY, base=FAKE):
    lay = kvm.kvm_layout_canonical(m.L, m.H, m.Hq, m.D, m.B, m.dtype, n_blocks)
    return kvm.Pool(base, n_blocks, lay)


def _einval(fn, *a, **kw):
    with pytest.raises(kvm.KvmError) as e:
        fn(*a, stream=0, **kw)
    assert e.value.status == kvm.KVM_EINVAL, e.value
    return e.value.detail


def test_argument_errors_come_before_any_launch():
    src, dst = _pool(), _pool(base=FAKE + (1 << 32))
    ok_s = kvm.Batch([0, 3], [5, 6, 7], [40], FAKE)
    ok_d = kvm.Batch([0, 3], [1, 2, 3], [40], FAKE)
    big = 1 << 30
    # k beyond the table, negative k
    assert "k[0]" in _einval(kvm.kvm_migrate, src, kvm.Batch([0, 3], [5, 6, 7], [49], FAKE), dst, ok_d)
    assert "k[0]" in _einval(kvm.kvm_pack, src, kvm.Batch([0, 3], [5, 6, 7], [-1], FAKE), FAKE, big)
    # block id outside the pool (only entries that hold tokens [0,k) are checked)
    assert "outside" in _einval(kvm.kvm_pack, src, kvm.Batch([0, 3], [5, 32, 7], [40], FAKE), FAKE, big)
    assert "outside" in _einval(kvm.kvm_unpack, FAKE, dst, kvm.Batch([0, 3], [5, -1, 7], [40], FAKE),
                                staging_bytes=big)
    # duplicate destination id
    assert "twice" in _einval(kvm.kvm_migrate, src, ok_s, dst, kvm.Batch([0, 3], [1, 2, 1], [40], FAKE))
    assert "twice" in _einval(kvm.kvm_unpack, FAKE, dst,
                              kvm.Batch([0, 2, 4], [1, 2, 3, 2], [20, 20], FAKE), staging_bytes=big)
    # batches that do not match
    assert "n_req" in _einval(kvm.kvm_migrate, src, ok_s, dst,
                              kvm.Batch([0, 3, 3], [1, 2, 3], [40, 0], FAKE))
    assert "k differs" in _einval(kvm.kvm_migrate, src, ok_s, dst, kvm.Batch([0, 3], [1, 2, 3], [39], FAKE))
    other = _pool(m=wl.Model("o", 2, 4, 4, 128, 16, "f16"), base=FAKE + (1 << 33))
    assert "layouts differ" in _einval(kvm.kvm_migrate, src, ok_s, other, ok_d)
    # staging buffer
    need = 40 * wl.TINY.bytes_per_token
    assert "too small" in _einval(kvm.kvm_pack, src, ok_s, FAKE, need - 1)
    assert "aligned" in _einval(kvm.kvm_pack, src, ok_s, FAKE + 8, need)
    assert "NULL" in _einval(kvm.kvm_unpack, None, dst, ok_d, staging_bytes=need)
    span = kvm.kvm_pool_span_bytes(src.layout, 32)
    assert "overlaps" in _einval(kvm.kvm_pack, src, ok_s, FAKE + span - 16, need)
    assert "overlaps" in _einval(kvm.kvm_unpack, FAKE + (1 << 32) - need + 16, dst, ok_d, staging_bytes=need)
    # pointers
    assert "base is NULL" in _einval(kvm.kvm_pack, _pool(base=None), ok_s, FAKE, big)
    assert "aligned" in _einval(kvm.kvm_pack, _pool(base=FAKE + 4), ok_s, FAKE, big)
    assert "bt_blocks_dev" in _einval(kvm.kvm_pack, src, kvm.Batch([0, 3], [5, 6, 7], [40], None), FAKE, big)
    # offsets
    bad = kvm.Batch([1, 3], [5, 6, 7], [20], FAKE)
    assert "bt_offsets[0]" in _einval(kvm.kvm_pack, src, bad, FAKE, big)
    bad = kvm.Batch([0, 3, 2], [5, 6, 7], [20, 0], FAKE)
    assert "non-decreasing" in _einval(kvm.kvm_pack, src, bad, FAKE, big)
    # in-pool migration: a block both read and written, overlapping but different pools
    assert "both read and written" in _einval(kvm.kvm_migrate, src, ok_s, src,
                                              kvm.Batch([0, 3], [1, 6, 3], [40], FAKE))
    assert "overlap" in _einval(kvm.kvm_migrate, src, ok_s, _pool(base=FAKE + 4096), ok_d)
    assert "host block ids" in _einval(kvm.kvm_migrate, src, ok_s, src,
                                       kvm.Batch([0, 3], [1, 2, 3], [40], FAKE, host_ids=False))
    # decode
    assert "q_dev" in _einval(kvm.kvm_paged_decode, src, ok_s, None, FAKE)
    assert "scale" in _einval(kvm.kvm_paged_decode, src, ok_s, FAKE, FAKE, scale=-1.0)
    odd = _pool(m=wl.Model("o", 2, 4, 4, 1024, 16, "f16"))
    assert "supported shapes" in _einval(kvm.kvm_paged_decode, odd, ok_s, FAKE, FAKE)


def test_empty_batches_are_no_ops_without_a_device():
    src, dst = _pool(), _pool(base=FAKE + (1 << 32))
    empty = kvm.Batch([0], [], [], None)
    assert kvm.kvm_migrate(src, empty, dst, empty, stream=0) == 0
    assert kvm.kvm_pack(src, empty, None, 0, stream=0) == 0
    zero = kvm.Batch([0, 2, 2], [3, 4], [0, 0], None)     # pure token-transfer requests
    assert kvm.kvm_migrate(src, zero, dst, zero, stream=0) == 0
    assert kvm.kvm_unpack(None, dst, zero, staging_bytes=0, stream=0) == 0
    assert kvm.kvm_paged_decode(src, zero, None, None, stream=0) == 0
    assert kvm.kvm_staging_bytes(src.layout, zero) == 0


def test_freelist_matches_oracle_allocator(oracle):
    rng = np.random.default_rng(0)
    for n in (1, 5, 16, 64, 65, 200):
        occ = (rng.random(n) < 0.4).astype(np.uint8)
        a, b = kvm.FreeList(n, occ), oracle.FreeList(n, occ)
        held = []
        for _ in range(60):
            assert a.available() == b.available()
            if held and rng.random() < 0.4:
                ids = held.pop(rng.integers(len(held)))
                a.free(ids); b.release(ids)
            else:
                want = int(rng.integers(0, n // 2 + 2))
                exp = b.alloc(want)
                if exp is None:
                    before = a.available()
                    with pytest.raises(kvm.KvmError) as e:
                        a.alloc(want)
                    assert e.value.status == kvm.KVM_ENOMEM and a.available() == before
                else:
                    got = a.alloc(want)
                    assert list(got) == exp
                    if want:
                        held.append(got)
    fl = kvm.FreeList(8, [1, 0, 0, 1, 0, 0, 0, 0])
    for bad in ([1], [0, 0], [8], [-1], [0, 3, 9]):
        before = fl.available()
        with pytest.raises(kvm.KvmError) as e:
            fl.free(bad)
        assert e.value.status == kvm.KVM_EINVAL and fl.available() == before
    assert list(fl.alloc(6)) == [1, 2, 4, 5, 6, 7]   # the failed frees changed nothing
    fl.free([0, 3])
    assert list(fl.alloc(2)) == [0, 3]
    # reserve takes named ids off the list, all-or-nothing
    fl = kvm.FreeList(8, [1, 0, 0, 1, 0, 0, 0, 0])
    fl.reserve([2, 6])
    assert fl.available() == 4 and list(fl.alloc(2)) == [1, 4]
    for bad in ([2], [0], [5, 5], [8], [7, 6]):
        before = fl.available()
        with pytest.raises(kvm.KvmError) as e:
            fl.reserve(bad)
        assert e.value.status == kvm.KVM_EINVAL and fl.available() == before
    assert list(fl.alloc(2)) == [5, 7]
    with pytest.raises(kvm.KvmError):
        kvm.FreeList(0)


def test_options_and_strerror():
    L = kvm.lib()
    assert L.kvm_strerror(0) == b"ok" and L.kvm_strerror(-2) == b"free list exhausted"
    for name, val in (("copy.order", 2), ("copy.nontemporal", 2), ("nope", 1), ("copy.unroll", 1),
                      ("decode.max_splits", 0), ("decode.force_splits", 65), ("decode.spread", 7),
                      ("decode.spread", -2)):
        with pytest.raises(kvm.KvmError):
            kvm.kvm_set_option(name, val)
    kvm.kvm_set_option("copy.order", -1)
    kvm.kvm_set_option("decode.force_splits", 0)
    kvm.kvm_set_option("decode.spread", 6)
    kvm.kvm_set_option("decode.spread", -1)


def test_per_request_limit_is_checked_before_the_first_launch():
    """65 requests, the last one beyond the per-call block limit: the error must come
    before the launch that would carry the first 64 (an error means nothing ran)."""
    n_big = 65536
    n_blocks = 64 + n_big
    src, dst = _pool(n_blocks), _pool(n_blocks, base=FAKE + (1 << 40))
    off = np.concatenate([np.arange(65), [64 + n_big]]).astype(np.int32)
    blk = np.arange(n_blocks, dtype=np.int32)
    k = np.array([16] * 64 + [n_big * 16], np.int32)
    b_s = kvm.Batch(off, blk, k, FAKE)
    b_d = kvm.Batch(off, blk, k, FAKE)
    assert "65535" in _einval(kvm.kvm_migrate, src, b_s, dst, b_d)
    assert "65535" in _einval(kvm.kvm_unpack, FAKE + (1 << 41), dst, b_d, staging_bytes=1 << 40)


def test_options_reset():
    kvm.kvm_set_option("copy.order", 0)
    kvm.kvm_set_option("decode.mfma", 1)
    kvm.kvm_set_option("reset", 0)
    # an out-of-range value is still refused, an unknown name too
    for name, v in (("copy.order", 3), ("decode.cap_waves", 5), ("no.such.option", 1)):
        with pytest.raises(kvm.KvmError) as e:
            kvm.kvm_set_option(name, v)
        assert e.value.status == kvm.KVM_EINVAL


def test_static_scratch_decode_rejects_a_plan_beyond_its_array():
    """kvm_paged_decode_static refuses, before any HIP call, a batch whose split
    workspace is larger than the static array; the constant matches the header."""
    text = open(os.path.join(ROOT, "include", "kvm.h")).read()
    mo = re.search(r"#define\s+KVM_STATIC_SCRATCH_BYTES\s+\((\d+)\s*<<\s*(\d+)\)", text)
    assert mo and int(mo.group(1)) << int(mo.group(2)) == kvm.KVM_STATIC_SCRATCH_BYTES
    m = wl.LLAMA3_8B
    pool = _pool(16 * 1024, m=m)
    off = (np.arange(17) * 1024).astype(np.int32)
    batch = kvm.Batch(off, np.arange(16 * 1024, dtype=np.int32), [16384] * 16, FAKE)
    try:
        kvm.kvm_set_option("decode.force_splits", 64)
        need = kvm.kvm_decode_workspace_bytes(pool.layout, batch)
        assert need == 16 * m.L * m.Hq * 64 * (m.D + 2) * 4 > kvm.KVM_STATIC_SCRATCH_BYTES
        detail = _einval(kvm.kvm_paged_decode_static, pool, batch, FAKE, FAKE)
        assert str(need) in detail and str(kvm.KVM_STATIC_SCRATCH_BYTES) in detail
    finally:
        kvm.kvm_set_option("reset", 0)
    # the same argument checks as kvm_paged_decode
    assert "q_dev" in _einval(kvm.kvm_paged_decode_static, pool, batch, None, FAKE)


def test_sequencer_host_logic_without_a_device():
    """kvm_sequencer_*: sizes, argument checks, all-or-nothing allocation and the return
    of destination blocks of orders that were staged but never enqueued.  Nothing is
    flushed here, so no HIP call is made."""
    L = kvm.lib()
    assert L.kvm_sequencer_table_ints(10, 16, 4) == (4 + 2) * 2 * 10 * 16
    assert L.kvm_sequencer_table_ints(0, 16, 4) == -1
    n = L.kvm_sequencer_table_ints(10, 4, 2)
    host = np.zeros(n, np.int32)
    assert not L.kvm_sequencer_create(10, 4, 2, None, FAKE, n, None, 0)
    assert not L.kvm_sequencer_create(10, 4, 2, host.ctypes.data, FAKE, n - 1, None, 0)
    assert b"table" in L.kvm_last_error()
    seq = L.kvm_sequencer_create(10, 4, 2, host.ctypes.data, FAKE, n, None, 0)
    assert seq
    src, dst = _pool(32), _pool(32, base=FAKE + (1 << 32))
    fs, fd = kvm.FreeList(32), kvm.FreeList(32, [1, 0, 1] + [0] * 29)
    table = np.array([3, 9, 4], np.int32)
    fs.reserve(table)
    out = np.full(4, -1, np.int32)

    def stage(k, tab=table, q=None, o=None, row=0, n_tab=None):
        return L.kvm_sequencer_stage(seq, ctypes.byref(src.c), fs._h, ctypes.byref(dst.c), fd._h,
                                     tab.ctypes.data, len(tab) if n_tab is None else n_tab, k, q, o, row,
                                     out.ctypes.data, None)

    assert stage(49) == kvm.KVM_EINVAL and stage(-1) == kvm.KVM_EINVAL          # k beyond the table
    assert stage(16, np.array([3, 32, 4], np.int32)) == kvm.KVM_EINVAL            # id outside the pool
    assert stage(16, q=FAKE, o=None) == kvm.KVM_EINVAL                            # decode without an output
    assert stage(16, np.arange(11, dtype=np.int32), n_tab=11) == kvm.KVM_EINVAL   # longer than max_blocks
    assert fd.available() == 30 and (out == -1).all()
    assert stage(40) == kvm.KVM_OK
    assert list(out[:3]) == [1, 3, 4] and fd.available() == 27                    # lowest free ids first
    assert stage(0) == kvm.KVM_OK and fd.available() == 27                        # a pure token-transfer order
    assert L.kvm_sequencer_launches(seq) == 0
    L.kvm_sequencer_destroy(seq)            # never enqueued: the destination blocks go back
    assert fd.available() == 30 and fs.available() == 29                          # ... the source stays allocated
