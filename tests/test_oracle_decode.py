"""Pins for the CPU oracle's paged decode attention and its 16-bit widening.

The paper (arXiv 2501.06709, Sec. "Background & Related Work") only says that
decoding reads the KV cache of all earlier tokens; the oracle is textbook
scaled-dot-product attention in fp64.  It is pinned by closed forms (one token,
zero query, a dominating key), by invariances (placement, GQA = MHA on repeated
heads), by numpy's own 16-bit conversions over all 65536 patterns, and by
torch's fp64 scaled_dot_product_attention on gathered contiguous K and V.
"""
import numpy as np
import pytest
import torch

import kvm_workload as wl


def view6(pool, m, n_blocks):
    return pool.reshape(m.L, 2, n_blocks, m.H, m.B, m.D)


def make_case(m, nblk, lens, seed):
    rng = np.random.default_rng(seed)
    pool = wl.gen_pool_host(seed, wl.STREAM_SRC, m, nblk)
    perm = rng.permutation(nblk)
    tabs, p = [], 0
    for ln in lens:
        n = -(-ln // m.B)
        tabs.append(perm[p:p + n].astype(np.int32)); p += n
    off = np.zeros(len(lens) + 1, np.int32)
    off[1:] = np.cumsum([len(t) for t in tabs])
    q = wl.gen_q(seed, m, len(lens))
    return pool, tabs, off, np.concatenate(tabs), q


def test_widen_matches_numpy_for_every_pattern(oracle):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    for dt in ("f16", "bf16"):
        ref = wl.bits16_to_f64(bits, dt)
        got = np.array([oracle.widen(b, dt) for b in bits])
        nan = np.isnan(ref)
        assert np.array_equal(np.isnan(got), nan)
        assert np.array_equal(got[~nan], ref[~nan])
        assert np.array_equal(np.signbit(got[~nan]), np.signbit(ref[~nan]))


@pytest.mark.parametrize("m", [wl.Model("mha", 2, 2, 2, 16, 4, "f16"),
                               wl.Model("gqa", 2, 2, 8, 16, 4, "bf16")])
def test_against_torch_sdpa_fp64(oracle, m):
    nblk, lens = 32, [1, 4, 5, 23, 16]
    pool, tabs, off, blk, q = make_case(m, nblk, lens, 11)
    st = oracle.canonical_strides(m.L, m.H, m.D, m.B, nblk)
    out = oracle.paged_decode(pool, st, m.L, m.H, m.Hq, m.D, m.B, m.dtype, off, blk, lens, q)
    p6 = wl.bits16_to_f64(view6(pool, m, nblk), m.dtype)
    qf = wl.bits16_to_f64(q, m.dtype)
    g = m.Hq // m.H
    for r, ln in enumerate(lens):
        kv = np.take(p6, tabs[r], axis=2).transpose(0, 1, 3, 2, 4, 5).reshape(m.L, 2, m.H, -1, m.D)
        kv = kv[:, :, :, :ln]
        K = torch.from_numpy(np.repeat(kv[:, 0], g, axis=1))   # [L][Hq][ln][D]
        V = torch.from_numpy(np.repeat(kv[:, 1], g, axis=1))
        Q = torch.from_numpy(qf[r])[:, :, None, :]             # [L][Hq][1][D]
        ref = torch.nn.functional.scaled_dot_product_attention(Q, K, V)[:, :, 0].numpy()
        assert np.allclose(out[r], ref, rtol=0, atol=1e-12), np.abs(out[r] - ref).max()


def test_closed_forms(oracle):
    m, nblk = wl.Model("c", 1, 2, 4, 8, 4, "f16"), 8
    pool, tabs, off, blk, q = make_case(m, nblk, [7], 12)
    st = oracle.canonical_strides(m.L, m.H, m.D, m.B, nblk)
    p6 = wl.bits16_to_f64(view6(pool, m, nblk), m.dtype)
    V = np.take(p6[0, 1], tabs[0], axis=0).transpose(1, 0, 2, 3).reshape(m.H, -1, m.D)  # [H][t][D]
    # one token: the output is that token's V row exactly, for the right KV head
    o1 = oracle.paged_decode(pool, st, m.L, m.H, m.Hq, m.D, m.B, m.dtype, off, blk, [1], q)
    for hq in range(m.Hq):
        assert np.array_equal(o1[0, 0, hq], V[hq // 2, 0])
    # zero query: uniform weights, the output is the mean of the V rows
    o0 = oracle.paged_decode(pool, st, m.L, m.H, m.Hq, m.D, m.B, m.dtype, off, blk, [7],
                             np.zeros_like(q))
    for hq in range(m.Hq):
        assert np.allclose(o0[0, 0, hq], V[hq // 2, :7].mean(axis=0), rtol=0, atol=1e-14)
    # scale = 0 does the same for any query; a huge scale picks the best-scoring key
    os0 = oracle.paged_decode(pool, st, m.L, m.H, m.Hq, m.D, m.B, m.dtype, off, blk, [7], q,
                              scale=0.0)
    assert np.allclose(os0, o0, rtol=0, atol=1e-14)
    K = np.take(p6[0, 0], tabs[0], axis=0).transpose(1, 0, 2, 3).reshape(m.H, -1, m.D)
    qf = wl.bits16_to_f64(q, m.dtype)
    big = oracle.paged_decode(pool, st, m.L, m.H, m.Hq, m.D, m.B, m.dtype, off, blk, [7], q,
                              scale=1e6)
    for hq in range(m.Hq):
        best = int(np.argmax(K[hq // 2, :7] @ qf[0, 0, hq]))
        assert np.allclose(big[0, 0, hq], V[hq // 2, best], rtol=0, atol=1e-9)
    # k = 0 leaves the output rows alone
    out = np.full((1, m.L, m.Hq, m.D), 7.0)
    oracle.paged_decode(pool, st, m.L, m.H, m.Hq, m.D, m.B, m.dtype, off, blk, [0], q, out=out)
    assert (out == 7.0).all()


def test_output_is_convex_combination_and_default_scale(oracle):
    m, nblk = wl.Model("c", 2, 2, 2, 16, 4, "bf16"), 16
    pool, tabs, off, blk, q = make_case(m, nblk, [30], 13)
    st = oracle.canonical_strides(m.L, m.H, m.D, m.B, nblk)
    out = oracle.paged_decode(pool, st, m.L, m.H, m.Hq, m.D, m.B, m.dtype, off, blk, [30], q)
    p6 = wl.bits16_to_f64(view6(pool, m, nblk), m.dtype)
    for l in range(m.L):
        V = np.take(p6[l, 1], tabs[0], axis=0).transpose(1, 0, 2, 3).reshape(m.H, -1, m.D)[:, :30]
        assert (out[0, l] <= V.max(axis=1) + 1e-12).all() and (out[0, l] >= V.min(axis=1) - 1e-12).all()
    explicit = oracle.paged_decode(pool, st, m.L, m.H, m.Hq, m.D, m.B, m.dtype, off, blk, [30], q,
                                   scale=1.0 / 4.0)  # 1/sqrt(16)
    assert np.array_equal(out, explicit)


def test_placement_invariance_and_gqa_equals_repeated_mha(oracle):
    m, nblk = wl.Model("g", 2, 2, 6, 8, 4, "f16"), 24
    pool, tabs, off, blk, q = make_case(m, nblk, [9, 14], 14)
    st = oracle.canonical_strides(m.L, m.H, m.D, m.B, nblk)
    out = oracle.paged_decode(pool, st, m.L, m.H, m.Hq, m.D, m.B, m.dtype, off, blk, [9, 14], q)
    # same logical KV in other physical blocks -> bit-identical fp64 result
    rng = np.random.default_rng(99)
    perm = rng.permutation(nblk)
    pool2 = np.zeros_like(pool)
    view6(pool2, m, nblk)[:, :, perm] = view6(pool, m, nblk)
    out2 = oracle.paged_decode(pool2, st, m.L, m.H, m.Hq, m.D, m.B, m.dtype, off,
                               perm[blk].astype(np.int32), [9, 14], q)
    assert np.array_equal(out, out2)
    # GQA with group 3 == MHA over a pool whose KV heads are each repeated 3 times
    mm = wl.Model("m", m.L, m.Hq, m.Hq, m.D, m.B, m.dtype)
    pool3 = np.repeat(view6(pool, m, nblk), m.Hq // m.H, axis=3).reshape(-1).copy()
    st3 = oracle.canonical_strides(mm.L, mm.H, mm.D, mm.B, nblk)
    out3 = oracle.paged_decode(pool3, st3, mm.L, mm.H, mm.Hq, mm.D, mm.B, mm.dtype, off, blk,
                               [9, 14], q)
    assert np.array_equal(out, out3)
    # attention over a migrated copy equals attention over the source
    dst = np.zeros_like(pool)
    d_tabs = np.arange(off[-1], dtype=np.int32)[::-1].copy()
    oracle.migrate(pool, st, dst, st, m.L, m.H, m.D, m.B, off, blk, off, d_tabs, [9, 14])
    out4 = oracle.paged_decode(dst, st, m.L, m.H, m.Hq, m.D, m.B, m.dtype, off, d_tabs, [9, 14], q)
    assert np.array_equal(out, out4)
