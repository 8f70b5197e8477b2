"""GPU parity: kvm_paged_decode through the C ABI against the fp64 CPU oracle.

Bar: inputs fp16 / bf16, fp32 accumulation, fp32 output within 2e-3 absolute of
the fp64 oracle.  A 16-bit output is compared with the oracle rounded to that
type with one unit in the last place of slack.  Decode over a migrated copy must
equal decode over the source bit for bit, because the kernel's reduction order
depends on logical token positions only.
"""
import numpy as np
import pytest
import torch

import kvm_workload as wl
import paper_2501_06709_amd as kvm

from gpu_util import DEV, Side, make_pair, to_dev, to_host

pytestmark = pytest.mark.gpu
TOL = 2e-3


def gpu_decode(side, q, out_f32=True, scale=0.0, workspace=True, batch=None):
    m = side.m
    batch = batch or side.batch
    q_dev = to_dev(q)
    out = torch.full(q.shape, 7.0, dtype=torch.float32, device=DEV) if out_f32 else \
        torch.zeros(q.shape, dtype=torch.int16, device=DEV)
    ws = None
    nbytes = kvm.kvm_decode_workspace_bytes(side.layout, batch)
    if workspace and nbytes > 0:
        ws = torch.empty(nbytes, dtype=torch.uint8, device=DEV)
    kvm.kvm_paged_decode(side.pool, batch, q_dev, out, out_is_f32=out_f32, scale=scale, workspace=ws)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def oracle_decode(orc, side, q, scale=None):
    m = side.m
    return orc.paged_decode(side.host, side.st, m.L, m.H, m.Hq, m.D, m.B, m.dtype, side.off,
                            side.blk, side.k, q, scale=scale)


SHAPES = [
    wl.Model("tiny", 2, 4, 4, 64, 16, "f16"),
    wl.Model("mha128", 2, 3, 3, 128, 16, "f16"),
    wl.Model("gqa4", 2, 2, 8, 128, 16, "bf16"),
    wl.Model("gqa2", 1, 2, 4, 64, 16, "bf16"),
    wl.Model("gqa8", 1, 1, 8, 128, 16, "f16"),
    wl.Model("gqa3", 1, 2, 6, 64, 16, "f16"),
]


VARIANTS = {"matrix_core_scores": 1, "vector_unit_scores": 0, "shipped": -1}


def set_variant(name):
    kvm.kvm_set_option("decode.mfma", VARIANTS[name])


@pytest.mark.parametrize("variant", list(VARIANTS))
@pytest.mark.parametrize("m", SHAPES, ids=[s.name for s in SHAPES])
def test_decode_matches_oracle(oracle, m, variant):
    """The grouped-query kernels (scores on the matrix cores or on the vector unit) and
    the MHA kernel against the fp64 oracle."""
    lens = [1, 15, 16, 17, 100, 333, 64]
    src, _ = make_pair(m, 64, 8, lens, [0] * len(lens), seed=21, finite=True)
    side = Side(m, 64, src.host, src.tables, lens)
    q = wl.gen_q(21, m, len(lens))
    try:
        set_variant(variant)
        got = gpu_decode(side, q)
    finally:
        set_variant("shipped")
    ref = oracle_decode(oracle, side, q)
    assert np.abs(got - ref).max() < TOL, np.abs(got - ref).max()


@pytest.mark.parametrize("variant", ["matrix_core_scores", "vector_unit_scores"])
@pytest.mark.parametrize("m", [SHAPES[1], SHAPES[2], SHAPES[4]], ids=["mha128", "gqa4", "gqa8"])
def test_every_context_length_up_to_nine_blocks(oracle, m, variant):
    """The kernels for head_dim 128 give each wave four token rows of every block and
    walk four blocks per step: every number of blocks modulo four and every fill of the
    last block must come out right, in both the capped and the uncapped instance."""
    lens = list(range(1, 9 * 16 + 2))
    n_blocks = sum(-(-k // 16) for k in lens)
    src, _ = make_pair(m, n_blocks + 8, 8, lens, [0] * len(lens), seed=31, finite=True)
    side = Side(m, n_blocks + 8, src.host, src.tables, lens)
    q = wl.gen_q(31, m, len(lens))
    ref = oracle_decode(oracle, side, q)
    try:
        set_variant(variant)
        for cap, spread in ((0, -1), (1, -1), (0, 0), (1, 1)):
            kvm.kvm_set_option("decode.cap_waves", cap)
            kvm.kvm_set_option("decode.spread", spread)
            got = gpu_decode(side, q)
            err = np.abs(got - ref).reshape(len(lens), -1).max(axis=1)
            assert err.max() < TOL, (cap, spread, int(err.argmax()) + 1, err.max())
    finally:
        kvm.kvm_set_option("decode.cap_waves", -1)
        kvm.kvm_set_option("decode.spread", -1)
        set_variant("shipped")


@pytest.mark.parametrize("variant", ["matrix_core_scores", "vector_unit_scores"])
@pytest.mark.parametrize("m", [SHAPES[1], SHAPES[2], SHAPES[4]], ids=["mha128", "gqa4", "gqa8"])
def test_interleaved_block_order_at_every_spread(oracle, m, variant):
    """A step of the head_dim-128 kernels reads four table entries that lie 2^spread
    entries apart (groups of 4 * 2^spread entries, the remainder with halved distances,
    the last entries in table order).  Contexts of 10 to 150 blocks with every kind of
    last block, every spread: each entry must be read exactly once, and the partly
    filled block last."""
    lens = [16 * n + r for n in range(10, 150, 9) for r in (0, 1, 15)] + [16 * 129 + 7, 16 * 64, 16 * 256]
    n_blocks = sum(-(-k // 16) for k in lens)
    src, _ = make_pair(m, n_blocks + 8, 8, lens, [0] * len(lens), seed=33, finite=True)
    side = Side(m, n_blocks + 8, src.host, src.tables, lens)
    q = wl.gen_q(33, m, len(lens))
    ref = oracle_decode(oracle, side, q)
    try:
        set_variant(variant)
        for spread in range(0, 7):
            kvm.kvm_set_option("decode.spread", spread)
            got = gpu_decode(side, q)
            err = np.abs(got - ref).reshape(len(lens), -1).max(axis=1)
            assert err.max() < TOL, (spread, lens[int(err.argmax())], err.max())
    finally:
        kvm.kvm_set_option("decode.spread", -1)
        set_variant("shipped")


def test_decode_k0_rows_untouched_and_scale(oracle):
    m = wl.Model("z", 2, 2, 4, 128, 16, "bf16")
    lens = [40, 20, 9]
    src, _ = make_pair(m, 16, 8, lens, [0, 0, 0], seed=22, finite=True)
    side = Side(m, 16, src.host, src.tables, [40, 0, 9])
    q = wl.gen_q(22, m, 3)
    got = gpu_decode(side, q, scale=0.3)
    ref = oracle_decode(oracle, side, q, scale=0.3)
    assert (got[1] == 7.0).all()
    assert np.abs(got[[0, 2]] - ref[[0, 2]]).max() < TOL


@pytest.mark.parametrize("variant", ["matrix_core_scores", "vector_unit_scores"])
def test_capped_occupancy_instances_give_the_same_bits(oracle, variant):
    """The kernels exist in two instances (at most two or eight waves per SIMD, chosen by
    mean context length); they are the same arithmetic."""
    outs = []
    for m in (SHAPES[1], SHAPES[2]):
        lens = [333, 17, 64]
        src, _ = make_pair(m, 64, 8, lens, [0] * len(lens), seed=29, finite=True)
        side = Side(m, 64, src.host, src.tables, lens)
        q = wl.gen_q(29, m, len(lens))
        ref = oracle_decode(oracle, side, q)
        try:
            set_variant(variant)
            for cap in (0, 1):
                kvm.kvm_set_option("decode.cap_waves", cap)
                outs.append(gpu_decode(side, q))
        finally:
            kvm.kvm_set_option("decode.cap_waves", -1)
            set_variant("shipped")
        assert np.array_equal(outs[-1], outs[-2])
        assert np.abs(outs[-1] - ref).max() < TOL


@pytest.mark.parametrize("splits", [2, 3, 7, 64])
def test_context_splits_match_unsplit_and_oracle(oracle, splits):
    m = wl.Model("sp", 2, 2, 8, 128, 16, "f16")
    lens = [700, 33, 250, 16]
    src, _ = make_pair(m, 80, 8, lens, [0] * 4, seed=23, finite=True)
    side = Side(m, 80, src.host, src.tables, lens)
    q = wl.gen_q(23, m, len(lens))
    ref = oracle_decode(oracle, side, q)
    try:
        kvm.kvm_set_option("decode.force_splits", splits)
        assert kvm.kvm_decode_workspace_bytes(side.layout, side.batch) == \
            len(lens) * m.L * m.Hq * splits * (m.D + 2) * 4
        got = gpu_decode(side, q)
        nows = gpu_decode(side, q, workspace=False)   # no workspace: falls back to one split
        kvm.kvm_set_option("decode.force_splits", 1)
        one = gpu_decode(side, q)
    finally:
        kvm.kvm_set_option("decode.force_splits", 0)
    assert np.abs(got - ref).max() < TOL and np.abs(one - ref).max() < TOL
    assert np.abs(got - one).max() < 1e-5
    assert np.array_equal(nows, one)


def test_sixteen_bit_output(oracle):
    for m in (wl.Model("h", 1, 2, 2, 128, 16, "f16"), wl.Model("b", 1, 2, 8, 128, 16, "bf16")):
        lens = [90, 5]
        src, _ = make_pair(m, 16, 8, lens, [0, 0], seed=24, finite=True)
        side = Side(m, 16, src.host, src.tables, lens)
        q = wl.gen_q(24, m, 2)
        got_bits = gpu_decode(side, q, out_f32=False).view(np.uint16)
        got = wl.bits16_to_f64(got_bits, m.dtype)
        ref = oracle_decode(oracle, side, q)
        mbits = 10 if m.dtype == "f16" else 7
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(ref), 2.0**-14))) - mbits)
        assert (np.abs(got - ref) <= ulp).all(), (np.abs(got - ref) / ulp).max()


def test_output_at_four_byte_alignment_gives_the_same_bits():
    """The output may start at any multiple of 4 bytes; the kernels then store dwords
    instead of 16-byte pieces.  Same bits, and nothing outside the rows is written."""
    for m in (wl.Model("h", 2, 2, 2, 128, 16, "f16"), wl.Model("b", 2, 2, 8, 128, 16, "bf16"),
              wl.Model("e", 1, 1, 8, 128, 16, "f16"), wl.Model("t", 2, 4, 4, 64, 16, "f16")):
        lens = [90, 5, 33]
        src, _ = make_pair(m, 16, 8, lens, [0, 0, 0], seed=27, finite=True)
        side = Side(m, 16, src.host, src.tables, lens)
        q = wl.gen_q(27, m, 3)
        q_dev = to_dev(q)
        n = int(np.prod(q.shape))
        for f32 in (True, False):
            dt = torch.float32 if f32 else torch.int16
            step = 1 if f32 else 2          # elements in 4 bytes
            ref = torch.zeros(n, dtype=dt, device=DEV)
            kvm.kvm_paged_decode(side.pool, side.batch, q_dev, ref, out_is_f32=f32)
            for shift in (1, 2, 3):
                buf = torch.full((n + 8 * step,), 5, dtype=dt, device=DEV)
                out = buf[shift * step: shift * step + n]
                assert out.data_ptr() % 16 == 4 * shift
                kvm.kvm_paged_decode(side.pool, side.batch, q_dev, out, out_is_f32=f32)
                torch.cuda.synchronize()
                assert torch.equal(out, ref), (m.name, f32, shift)
                assert (buf[:shift * step] == 5).all() and (buf[shift * step + n:] == 5).all()


def test_garbage_beyond_the_context_is_ignored(oracle):
    """Slots >= k of the last block and blocks past it may hold NaN patterns."""
    m = wl.Model("nan", 1, 2, 4, 128, 16, "bf16")
    lens, ks = [48, 40], [37, 16]
    src, _ = make_pair(m, 16, 8, lens, [0, 0], seed=26, finite=True)
    host = src.host.copy()
    p6 = host.reshape(m.L, 2, 16, m.H, m.B, m.D)
    for tab, k in zip(src.tables, ks):
        for j, b in enumerate(tab):
            p6[:, :, b, :, max(0, min(m.B, k - j * m.B)):] = 0x7FFF
    side = Side(m, 16, host, src.tables, ks)
    clean = Side(m, 16, src.host, src.tables, ks)
    q = wl.gen_q(26, m, 2)
    got = gpu_decode(side, q)
    assert np.array_equal(got, gpu_decode(clean, q))
    assert np.abs(got - oracle_decode(oracle, clean, q)).max() < TOL


def test_decode_after_migration_is_bitwise_the_same(oracle):
    """The usability proof: attention over the destination cache equals attention
    over the first k tokens of the source cache."""
    m = wl.LLAMA3_8B
    m = wl.Model("8b4", 4, m.H, m.Hq, m.D, m.B, m.dtype)
    lens, ks = [300, 49, 130], [225, 36, 97]
    src, dst = make_pair(m, 48, 48, lens, ks, seed=25, finite=True)
    kvm.kvm_migrate(src.pool, src.batch, dst.pool, dst.batch)
    q = wl.gen_q(25, m, len(ks))
    a = gpu_decode(src, q)
    b = gpu_decode(dst, q)
    assert np.array_equal(a, b)
    ref = oracle_decode(oracle, src, q)
    assert np.abs(a - ref).max() < TOL
    # strided (token-major, padded) pool holding the same logical cache
    slot = m.H * m.D + 8
    tm = np.array([2 * m.B * slot, m.B * slot, m.L * 2 * m.B * slot, m.D, slot], dtype=np.int64)
    alt_host = np.zeros(wl.pool_span_elems(m, 48, tm), dtype=np.uint16)
    alt = Side(m, 48, alt_host, dst.tables, ks, strides=tm)
    kvm.kvm_migrate(src.pool, src.batch, alt.pool, alt.batch)
    c = gpu_decode(alt, q)
    assert np.array_equal(a, c)


GENERIC = [
    wl.Model("d80", 2, 2, 4, 80, 16, "f16"),      # head_dim not a power of two
    wl.Model("d256", 1, 2, 2, 256, 16, "bf16"),
    wl.Model("b8", 2, 3, 3, 64, 8, "bf16"),       # other block sizes
    wl.Model("b32", 1, 2, 6, 128, 32, "f16"),
    wl.Model("d512", 1, 1, 2, 512, 4, "f16"),
]


@pytest.mark.parametrize("m", GENERIC, ids=[s.name for s in GENERIC])
def test_fallback_kernel_for_other_shapes(oracle, m):
    lens = [1, m.B - 1, m.B, m.B + 1, 5 * m.B + 3, 150]
    src, _ = make_pair(m, 64, 8, lens, [0] * len(lens), seed=27, finite=True)
    side = Side(m, 64, src.host, src.tables, [lens[0], 0] + lens[2:])
    q = wl.gen_q(27, m, len(lens))
    got = gpu_decode(side, q)
    ref = oracle_decode(oracle, side, q)
    assert (got[1] == 7.0).all()
    keep = [0, 2, 3, 4, 5]
    assert np.abs(got[keep] - ref[keep]).max() < TOL
    got16 = wl.bits16_to_f64(gpu_decode(side, q, out_f32=False).view(np.uint16), m.dtype)
    assert np.abs(got16[keep] - ref[keep]).max() < 0.05


def test_decode_rows_place_queries_and_outputs(oracle):
    """kvm_paged_decode_rows: request r reads q row rows[r] and writes out row rows[r];
    other rows of the output stay as they were; same bits as the identity call."""
    m = wl.Model("gqa4", 2, 2, 8, 128, 16, "bf16")
    lens = [100, 0, 333, 17]
    src, _ = make_pair(m, 64, 8, [max(x, 1) for x in lens], [0] * 4, seed=31, finite=True)
    side = Side(m, 64, src.host, src.tables, lens)
    rows = np.array([5, 2, 0, 9], np.int32)            # row 2 belongs to the k = 0 request
    q_small = wl.gen_q(31, m, 4)
    q_big = np.zeros((12,) + q_small.shape[1:], np.uint16)
    q_big[rows] = q_small
    ref = gpu_decode(side, q_small)                    # identity rows
    out = torch.full(q_big.shape, 7.0, dtype=torch.float32, device=DEV)
    kvm.kvm_paged_decode_rows(side.pool, side.batch, rows, to_dev(q_big), out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    for r in (0, 2, 3):
        assert np.array_equal(got[rows[r]], ref[r])
    untouched = [i for i in range(12) if i not in (5, 0, 9)]
    assert (got[untouched] == 7.0).all()
    exp = oracle_decode(oracle, side, q_small)
    assert np.abs(got[rows[[0, 2, 3]]] - exp[[0, 2, 3]]).max() < TOL
    # long contexts: the split workspace is indexed by position in the batch, not by row
    lens = [2500, 1800]
    src, _ = make_pair(m, 300, 8, lens, [0] * 2, seed=32, finite=True)
    side = Side(m, 300, src.host, src.tables, lens)
    q_small = wl.gen_q(32, m, 2)
    ref = gpu_decode(side, q_small)
    rows = np.array([40, 3], np.int32)
    q_big = np.zeros((41,) + q_small.shape[1:], np.uint16)
    q_big[rows] = q_small
    nws = kvm.kvm_decode_workspace_bytes(side.layout, side.batch)
    assert nws > 0
    ws = torch.empty(nws, dtype=torch.uint8, device=DEV)
    out = torch.full(q_big.shape, 7.0, dtype=torch.float32, device=DEV)
    kvm.kvm_paged_decode_rows(side.pool, side.batch, rows, to_dev(q_big), out, workspace=ws)
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy()[rows], ref)
    with pytest.raises(kvm.KvmError):
        kvm.kvm_paged_decode_rows(side.pool, side.batch, [3, 3], to_dev(q_big), out)
