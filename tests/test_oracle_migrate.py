"""Pins for the CPU oracle's pack / unpack / migrate and its allocator.

Nothing here compares the oracle with itself through the same formula: the
checks are invariants the problem fixes, special cases that reduce to numpy
library routines (take / slicing / array_equal), a hand-worked fixture of the
staging format, the paper's worked KV size, algebraic identities and brute
force over tiny inputs.  Citations: arXiv 2501.06709, Sec. "Background &
Related Work" (paged KV), Sec. "Motivation" Finding 4 (append-only prefix),
Sec. "Adaptive Request Migration" (source kept until transfer completes),
Sec. "System Model" (size linear in tokens).
"""
import itertools
import os

import numpy as np
import pytest

import kvm_workload as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def view6(pool, m, n_blocks):
    """Dense pool as [L][2][block][H][B][D] (numpy view, library indexing)."""
    return pool.reshape(m.L, 2, n_blocks, m.H, m.B, m.D)


def logical(pool, m, n_blocks, table, k):
    """Tokens [0,k) of a request as [L][2][H][k][D] using numpy take/transpose."""
    nb = -(-k // m.B)
    g = np.take(view6(pool, m, n_blocks), np.asarray(table[:nb], dtype=np.int64), axis=2)
    g = g.transpose(0, 1, 3, 2, 4, 5).reshape(m.L, 2, m.H, nb * m.B, m.D)
    return g[:, :, :, :k]


def csr(tables):
    off = np.zeros(len(tables) + 1, dtype=np.int32)
    off[1:] = np.cumsum([len(t) for t in tables])
    return off, (np.concatenate(tables).astype(np.int32) if tables else np.zeros(0, np.int32))


def random_pool(rng, m, n_blocks):
    return rng.integers(0, 65536, size=m.L * 2 * n_blocks * m.H * m.B * m.D).astype(np.uint16)


def tiny_case(oracle):
    w = wl.make("tiny")
    m = w.model
    src = wl.gen_pool_host(w.seed, wl.STREAM_SRC, m, w.n_blocks_src)
    dst = wl.gen_pool_host(w.seed, wl.STREAM_DST, m, w.n_blocks_dst)
    fl = oracle.FreeList(w.n_blocks_dst, w.dst_occupied)
    dst_tabs = [np.array(fl.alloc(n), dtype=np.int32) for n in w.n_dst_blocks()]
    return w, m, src, dst, dst_tabs


# --- closed forms -----------------------------------------------------------

def test_kv_size_matches_paper_worked_value(oracle):
    cfg = {}
    for line in open(os.path.join(GOLDEN, "kv_size_13b.txt")):
        if not line.startswith("#") and line.strip():
            key, val = line.split()
            cfg[key] = float(val)
    bpt = oracle.bytes_per_token(int(cfg["layers"]), int(cfg["kv_heads"]), int(cfg["head_dim"]))
    assert bpt == 819200
    size = bpt * int(cfg["tokens"])
    # "about 3.2 GB": within 5 % whether GB means 1e9 or 2^30 bytes
    assert abs(size / 1e9 - cfg["kv_size_about_gb"]) / cfg["kv_size_about_gb"] < 0.05
    assert abs(size / 2**30 - cfg["kv_size_about_gb"]) / cfg["kv_size_about_gb"] < 0.05
    # weights + 5 requests fit in the GPU, 6 do not (a dropped factor 2 for K and
    # V, or 4-byte elements, changes this count)
    assert int((cfg["gpu_gb"] - cfg["weights_gb"]) // (size / 2**30)) == int(cfg["max_batch"])


@pytest.mark.parametrize("m", [wl.TINY, wl.LLAMA2_7B, wl.LLAMA3_8B, wl.LLAMA2_13B])
def test_bytes_per_token_table(oracle, m):
    expect = {"tiny": 2048, "llama2_7b": 524288, "llama3_8b_gqa": 131072, "llama2_13b": 819200}
    assert oracle.bytes_per_token(m.L, m.H, m.D) == expect[m.name] == m.bytes_per_token


def test_staging_is_linear_in_k(oracle):
    m = wl.TINY
    for k in (0, 1, 15, 16, 17, 100):
        assert oracle.staging_elems(m.L, m.H, m.D, [k]) * 2 == k * m.bytes_per_token
    assert oracle.staging_elems(m.L, m.H, m.D, [3, 5, 0, 9]) * 2 == 17 * m.bytes_per_token


# --- hand-worked staging format ---------------------------------------------

def test_pack_format_golden(oracle):
    rows = [list(map(int, ln.split())) for ln in open(os.path.join(GOLDEN, "pack_format_small.txt"))
            if ln.strip() and not ln.startswith("#")]
    expect = np.array(rows, dtype=np.uint16).reshape(-1)
    L, H, B, D, nblk = 1, 2, 2, 2, 2
    kv, b, h, s, d = np.meshgrid(np.arange(2), np.arange(nblk), np.arange(H), np.arange(B),
                                 np.arange(D), indexing="ij")
    pool = (kv * 1000 + b * 100 + h * 10 + s * 2 + d + 1).astype(np.uint16).reshape(-1)
    st = oracle.canonical_strides(L, H, D, B, nblk)
    stage = oracle.pack(pool, st, L, H, D, B, [0, 2], [1, 0], [3])
    assert np.array_equal(stage, expect)
    # and unpack puts exactly those values back at the same places
    dst = np.zeros_like(pool)
    oracle.unpack(stage, dst, st, L, H, D, B, [0, 2], [1, 0], [3])
    mask = np.isin(pool, expect)
    assert np.array_equal(dst[mask], pool[mask]) and not dst[~mask].any()


# --- invariants on the tiny benchmark config ----------------------------------

def test_tiny_migrate_invariants(oracle):
    w, m, src, dst, dst_tabs = tiny_case(oracle)
    src0, dst0 = src.copy(), dst.copy()
    s_off, s_blk = w.src_csr()
    d_off, d_blk = csr(dst_tabs)
    oracle.migrate(src, oracle.canonical_strides(m.L, m.H, m.D, m.B, w.n_blocks_src), dst,
                   oracle.canonical_strides(m.L, m.H, m.D, m.B, w.n_blocks_dst),
                   m.L, m.H, m.D, m.B, s_off, s_blk, d_off, d_blk, w.k)
    # (iv) the source pool is never written
    assert np.array_equal(src, src0)
    # (i) every token lands bit-identical at its logical position
    for i, r in enumerate(w.migrate_ids):
        a = logical(src, m, w.n_blocks_src, w.src_tables[r], int(w.k[i]))
        b = logical(dst, m, w.n_blocks_dst, dst_tabs[i], int(w.k[i]))
        assert a.shape[3] == w.k[i] and np.array_equal(a, b)
    # (ii) destination blocks == the ids the allocator handed out == lowest free ids
    assert np.array_equal(d_blk, np.arange(len(d_blk)))
    changed = np.any(view6(dst, m, w.n_blocks_dst) != view6(dst0, m, w.n_blocks_dst),
                     axis=(0, 1, 3, 4, 5))
    assert set(np.nonzero(changed)[0]) == set(d_blk.tolist())
    # (iii) bytes outside the written slots are unchanged
    keep = np.ones(dst.shape, dtype=bool)
    k6 = view6(keep, m, w.n_blocks_dst)
    for i in range(len(w.k)):
        for j, b in enumerate(dst_tabs[i]):
            k6[:, :, b, :, :min(m.B, int(w.k[i]) - j * m.B)] = False
    assert np.array_equal(dst[keep], dst0[keep])
    assert keep.sum() == dst.size - int(w.k.sum()) * m.bytes_per_token // 2


def test_identity_table_is_a_slice_copy(oracle):
    m, nblk, nb = wl.Model("t", 3, 2, 2, 8, 4, "f16"), 10, 6
    rng = np.random.default_rng(1)
    src, dst = random_pool(rng, m, nblk), random_pool(rng, m, nblk)
    dst0 = dst.copy()
    st = oracle.canonical_strides(m.L, m.H, m.D, m.B, nblk)
    ident = np.arange(nb, dtype=np.int32)
    oracle.migrate(src, st, dst, st, m.L, m.H, m.D, m.B, [0, nb], ident, [0, nb], ident, [nb * m.B])
    assert np.array_equal(view6(dst, m, nblk)[:, :, :nb], view6(src, m, nblk)[:, :, :nb])
    assert np.array_equal(view6(dst, m, nblk)[:, :, nb:], view6(dst0, m, nblk)[:, :, nb:])
    # staging of an identity table with one head is the pool slice itself
    m1 = wl.Model("t1", 2, 1, 1, 8, 4, "f16")
    src1 = random_pool(rng, m1, nblk)
    st1 = oracle.canonical_strides(m1.L, m1.H, m1.D, m1.B, nblk)
    stage = oracle.pack(src1, st1, m1.L, m1.H, m1.D, m1.B, [0, nb], ident, [nb * m1.B])
    assert np.array_equal(stage.reshape(m1.L, 2, nb * m1.B * m1.D),
                          view6(src1, m1, nblk)[:, :, :nb].reshape(m1.L, 2, -1))


def test_permuted_destination_is_index_select(oracle):
    m, nblk = wl.Model("t", 2, 3, 3, 8, 4, "bf16"), 12
    rng = np.random.default_rng(2)
    src, dst = random_pool(rng, m, nblk), np.zeros(m.L * 2 * nblk * m.H * m.B * m.D, np.uint16)
    st = oracle.canonical_strides(m.L, m.H, m.D, m.B, nblk)
    sperm, dperm = rng.permutation(nblk).astype(np.int32), rng.permutation(nblk).astype(np.int32)
    oracle.migrate(src, st, dst, st, m.L, m.H, m.D, m.B, [0, nblk], sperm, [0, nblk], dperm,
                   [nblk * m.B])
    expect = np.zeros_like(view6(dst, m, nblk))
    expect[:, :, dperm] = np.take(view6(src, m, nblk), sperm, axis=2)
    assert np.array_equal(view6(dst, m, nblk), expect)


# --- algebra -------------------------------------------------------------------

def _small_batch(rng, m, nblk, lens, ks):
    perm_s, perm_d = rng.permutation(nblk), rng.permutation(nblk)
    s_tabs, d_tabs, p, q = [], [], 0, 0
    for ln, k in zip(lens, ks):
        n, nd = -(-ln // m.B), -(-k // m.B)
        s_tabs.append(perm_s[p:p + n].astype(np.int32)); p += n
        d_tabs.append(perm_d[q:q + nd].astype(np.int32)); q += nd
    return s_tabs, d_tabs


def test_unpack_of_pack_equals_migrate_and_batch_equals_singles(oracle):
    m, nblk = wl.Model("t", 2, 2, 4, 16, 4, "f16"), 40
    rng = np.random.default_rng(3)
    lens, ks = [13, 4, 1, 22, 9], [13, 3, 0, 17, 8]
    s_tabs, d_tabs = _small_batch(rng, m, nblk, lens, ks)
    src, dst0 = random_pool(rng, m, nblk), random_pool(rng, m, nblk)
    st = oracle.canonical_strides(m.L, m.H, m.D, m.B, nblk)
    s_off, s_blk = csr(s_tabs)
    d_off, d_blk = csr(d_tabs)
    a = dst0.copy()
    oracle.migrate(src, st, a, st, m.L, m.H, m.D, m.B, s_off, s_blk, d_off, d_blk, ks)
    b = dst0.copy()
    stage = oracle.pack(src, st, m.L, m.H, m.D, m.B, s_off, s_blk, ks)
    assert stage.size * 2 == sum(ks) * m.bytes_per_token
    oracle.unpack(stage, b, st, m.L, m.H, m.D, m.B, d_off, d_blk, ks)
    assert np.array_equal(a, b)
    c = dst0.copy()
    for r in (3, 0, 4, 1, 2):  # requests are independent: any order, one at a time
        oracle.migrate(src, st, c, st, m.L, m.H, m.D, m.B, [0, len(s_tabs[r])], s_tabs[r],
                       [0, len(d_tabs[r])], d_tabs[r], [ks[r]])
    assert np.array_equal(a, c)
    # layer ranges compose (used to spread the oracle over threads)
    e = dst0.copy()
    for lr in ((1, 2), (0, 1)):
        oracle.migrate(src, st, e, st, m.L, m.H, m.D, m.B, s_off, s_blk, d_off, d_blk, ks,
                       layers=lr)
    assert np.array_equal(a, e)


def test_round_trip_restores_logical_content(oracle):
    m, nblk = wl.Model("t", 2, 2, 2, 8, 4, "f16"), 16
    rng = np.random.default_rng(4)
    a, b, a2 = random_pool(rng, m, nblk), random_pool(rng, m, nblk), random_pool(rng, m, nblk)
    st = oracle.canonical_strides(m.L, m.H, m.D, m.B, nblk)
    ta, tb, ta2 = (rng.permutation(nblk)[:5].astype(np.int32) for _ in range(3))
    k = 18
    oracle.migrate(a, st, b, st, m.L, m.H, m.D, m.B, [0, 5], ta, [0, 5], tb, [k])
    oracle.migrate(b, st, a2, st, m.L, m.H, m.D, m.B, [0, 5], tb, [0, 5], ta2, [k])
    assert np.array_equal(logical(a, m, nblk, ta, k), logical(a2, m, nblk, ta2, k))


def test_prefix_property(oracle):
    """Append-only cache: moving [0,k) then [0,k') equals moving [0,k') once, and
    the staging of k is a per-(layer,kv,head) prefix of the staging of k'."""
    m, nblk = wl.Model("t", 2, 3, 3, 8, 4, "f16"), 16
    rng = np.random.default_rng(5)
    src, dst0 = random_pool(rng, m, nblk), random_pool(rng, m, nblk)
    st = oracle.canonical_strides(m.L, m.H, m.D, m.B, nblk)
    ts, td = rng.permutation(nblk)[:6].astype(np.int32), rng.permutation(nblk)[:6].astype(np.int32)
    k, k2 = 9, 22
    a, b = dst0.copy(), dst0.copy()
    oracle.migrate(src, st, a, st, m.L, m.H, m.D, m.B, [0, 6], ts, [0, 6], td, [k])
    oracle.migrate(src, st, a, st, m.L, m.H, m.D, m.B, [0, 6], ts, [0, 6], td, [k2])
    oracle.migrate(src, st, b, st, m.L, m.H, m.D, m.B, [0, 6], ts, [0, 6], td, [k2])
    assert np.array_equal(a, b)
    p1 = oracle.pack(src, st, m.L, m.H, m.D, m.B, [0, 6], ts, [k]).reshape(m.L, 2, m.H, k, m.D)
    p2 = oracle.pack(src, st, m.L, m.H, m.D, m.B, [0, 6], ts, [k2]).reshape(m.L, 2, m.H, k2, m.D)
    assert np.array_equal(p1, p2[:, :, :, :k])
    assert np.array_equal(p2, logical(src, m, nblk, ts, k2))


def test_strided_layouts_hold_the_same_logical_content(oracle):
    """A token-major block layout and a padded one are descriptor changes only."""
    m, nblk = wl.Model("t", 2, 3, 3, 8, 4, "f16"), 9
    rng = np.random.default_rng(6)
    dense = random_pool(rng, m, nblk)
    st = oracle.canonical_strides(m.L, m.H, m.D, m.B, nblk)
    # token-major: pool[block][layer][kv][slot][head][dim], plus 8 elements of padding per slot row
    slot = m.H * m.D + 8
    st2 = np.array([2 * m.B * slot, m.B * slot, m.L * 2 * m.B * slot, m.D, slot], dtype=np.int64)
    alt = np.zeros(nblk * m.L * 2 * m.B * slot, dtype=np.uint16)
    ident = np.arange(nblk, dtype=np.int32)
    oracle.migrate(dense, st, alt, st2, m.L, m.H, m.D, m.B, [0, nblk], ident, [0, nblk], ident,
                   [nblk * m.B])
    a6 = alt.reshape(nblk, m.L, 2, m.B, slot)[..., :m.H * m.D].reshape(nblk, m.L, 2, m.B, m.H, m.D)
    assert np.array_equal(a6.transpose(1, 2, 0, 4, 3, 5), view6(dense, m, nblk))
    assert not alt.reshape(nblk, m.L, 2, m.B, slot)[..., m.H * m.D:].any()
    # and a partial migration out of the strided pool gives the dense answer
    ts, td, k = np.array([7, 2, 5], np.int32), np.array([1, 8, 0], np.int32), 10
    out1, out2 = np.zeros_like(dense), np.zeros_like(dense)
    oracle.migrate(alt, st2, out1, st, m.L, m.H, m.D, m.B, [0, 3], ts, [0, 3], td, [k])
    oracle.migrate(dense, st, out2, st, m.L, m.H, m.D, m.B, [0, 3], ts, [0, 3], td, [k])
    assert np.array_equal(out1, out2)
    stage1 = oracle.pack(alt, st2, m.L, m.H, m.D, m.B, [0, 3], ts, [k])
    assert np.array_equal(stage1.reshape(m.L, 2, m.H, k, m.D), logical(dense, m, nblk, ts, k))


# --- brute force ------------------------------------------------------------------

def test_brute_force_all_k_and_all_permutations(oracle):
    m = wl.Model("bf", 2, 1, 1, 8, 4, "f16")
    rng = np.random.default_rng(7)
    nblk = 12
    st = oracle.canonical_strides(m.L, m.H, m.D, m.B, nblk)
    src, dst0 = random_pool(rng, m, nblk), random_pool(rng, m, nblk)
    # every k for a 48-token request
    ts, td = rng.permutation(nblk).astype(np.int32), rng.permutation(nblk).astype(np.int32)
    for k in range(0, 49):
        dst = dst0.copy()
        oracle.migrate(src, st, dst, st, m.L, m.H, m.D, m.B, [0, 12], ts, [0, 12], td, [k])
        if k:
            assert np.array_equal(logical(src, m, nblk, ts, k), logical(dst, m, nblk, td, k))
        assert int((dst != dst0).sum()) <= k * m.bytes_per_token // 2
        untouched = np.ones(dst.size, bool)
        u6 = view6(untouched, m, nblk)
        for j in range(-(-k // m.B)):
            u6[:, :, td[j], :, :min(m.B, k - j * m.B)] = False
        assert np.array_equal(dst[untouched], dst0[untouched])
    # every placement of up to 4 blocks in a 4-block pool, both sides
    nblk = 4
    st = oracle.canonical_strides(m.L, m.H, m.D, m.B, nblk)
    src, dst0 = random_pool(rng, m, nblk), random_pool(rng, m, nblk)
    for nb in range(1, 5):
        for ps in itertools.permutations(range(4), nb):
            for pd in itertools.permutations(range(4), nb):
                k = nb * m.B - 1
                dst = dst0.copy()
                oracle.migrate(src, st, dst, st, m.L, m.H, m.D, m.B, [0, nb],
                               np.array(ps, np.int32), [0, nb], np.array(pd, np.int32), [k])
                assert np.array_equal(logical(src, m, nblk, ps, k), logical(dst, m, nblk, pd, k))
                rest = [b for b in range(4) if b not in pd]
                assert np.array_equal(view6(dst, m, nblk)[:, :, rest], view6(dst0, m, nblk)[:, :, rest])
                last = view6(dst, m, nblk)[:, :, pd[-1], :, m.B - 1]
                assert np.array_equal(last, view6(dst0, m, nblk)[:, :, pd[-1], :, m.B - 1])


# --- token ranges (rounds of a live migration) ----------------------------------

def test_ranges_compose_and_touch_only_their_slots(oracle):
    m = wl.Model("rg", 2, 2, 2, 8, 4, "f16")
    rng = np.random.default_rng(8)
    nblk, ln = 12, 40
    st = oracle.canonical_strides(m.L, m.H, m.D, m.B, nblk)
    src, dst0 = random_pool(rng, m, nblk), random_pool(rng, m, nblk)
    ts, td = rng.permutation(nblk)[:10].astype(np.int32), rng.permutation(nblk)[:10].astype(np.int32)
    whole = {}
    for b in range(0, ln + 1):
        d = dst0.copy()
        oracle.migrate(src, st, d, st, m.L, m.H, m.D, m.B, [0, 10], ts, [0, 10], td, [b])
        whole[b] = d
    for a in range(0, ln + 1, 3):
        for b in range(a, ln + 1):
            # [0,a) then [a,b) leaves the destination as [0,b) at once
            d = whole[a].copy()
            oracle.migrate(src, st, d, st, m.L, m.H, m.D, m.B, [0, 10], ts, [0, 10], td, [b], start=[a])
            assert np.array_equal(d, whole[b]), (a, b)
            # the range alone writes exactly the slots of tokens [a,b)
            d = dst0.copy()
            oracle.migrate(src, st, d, st, m.L, m.H, m.D, m.B, [0, 10], ts, [0, 10], td, [b], start=[a])
            touched = np.zeros(d.size, bool)
            t6 = view6(touched, m, nblk)
            for t in range(a, b):
                t6[:, :, td[t // m.B], :, t % m.B] = True
            assert np.array_equal(d[~touched], dst0[~touched])
            assert np.array_equal(d[touched], whole[b][touched])
            # staging of the range is the slice [a,b) of the logical view, and unpack inverts it
            stage = oracle.pack(src, st, m.L, m.H, m.D, m.B, [0, 10], ts, [b], start=[a])
            assert stage.size * 2 == (b - a) * m.bytes_per_token
            if b > a:
                assert np.array_equal(stage.reshape(m.L, 2, m.H, b - a, m.D),
                                      logical(src, m, nblk, ts, b)[:, :, :, a:])
            e = dst0.copy()
            oracle.unpack(stage, e, st, m.L, m.H, m.D, m.B, [0, 10], td, [b], start=[a])
            assert np.array_equal(e, d)
    # batches: per-request ranges, staging concatenated in batch order
    ks, ss = [17, 9, 14], [5, 9, 0]
    s_tabs, d_tabs = _small_batch(rng, m, nblk, [17, 9, 14], ks)
    s_off, s_blk = csr(s_tabs)
    d_off, d_blk = csr(d_tabs)
    stage = oracle.pack(src, st, m.L, m.H, m.D, m.B, s_off, s_blk, ks, start=ss)
    parts = [oracle.pack(src, st, m.L, m.H, m.D, m.B, [0, len(t)], t, [k], start=[s0])
             for t, k, s0 in zip(s_tabs, ks, ss)]
    assert np.array_equal(stage, np.concatenate(parts))


# --- allocator -----------------------------------------------------------------

def test_freelist_brute_force(oracle):
    for n in range(1, 9):
        for mask in range(1 << n):
            occ = [(mask >> b) & 1 for b in range(n)]
            free_ids = [b for b in range(n) if not occ[b]]
            for want in range(0, n + 2):
                fl = oracle.FreeList(n, occ)
                got = fl.alloc(want)
                if want > len(free_ids):
                    assert got is None and fl.available() == len(free_ids)
                else:
                    assert got == free_ids[:want]
                    assert fl.available() == len(free_ids) - want
                    fl.release(got)
                    assert fl.available() == len(free_ids)
                    assert fl.alloc(len(free_ids)) == free_ids
    fl = oracle.FreeList(4, [1, 0, 0, 1])
    with pytest.raises(ValueError):
        fl.release([1])          # already free
    with pytest.raises(ValueError):
        fl.release([0, 0])       # repeated
    with pytest.raises(ValueError):
        fl.release([4])          # out of range
