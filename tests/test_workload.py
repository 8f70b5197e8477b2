"""The synthetic input generator: statistics, determinism and config structure."""
import numpy as np
import pytest

import kvm_workload as wl


def test_values_are_standard_normal_like_and_deterministic():
    w = np.arange(1 << 16, dtype=np.uint32)
    for dt in ("f16", "bf16"):
        bits = wl.gen_values(7, wl.STREAM_SRC, 3, 11, w, dt)
        v = wl.bits16_to_f64(bits, dt)
        assert abs(v.mean()) < 0.02 and abs(v.std() - 1.0) < 0.02
        assert np.abs(v).max() < 4.9 and (np.abs(v) > 2.5).any()
        assert np.array_equal(bits, wl.gen_values(7, wl.STREAM_SRC, 3, 11, w, dt))
    a = wl.gen_values(7, wl.STREAM_SRC, 3, 11, w, "f16")
    for other in (wl.gen_values(8, wl.STREAM_SRC, 3, 11, w, "f16"),
                  wl.gen_values(7, wl.STREAM_DST, 3, 11, w, "f16"),
                  wl.gen_values(7, wl.STREAM_SRC, 4, 11, w, "f16"),
                  wl.gen_values(7, wl.STREAM_SRC, 3, 12, w, "f16")):
        assert (a != other).mean() > 0.9


def test_rounding_to_16_bits_is_nearest_even():
    f = np.array([1.0, 1.0 + 2**-8, 1.0 + 3 * 2**-8, -1.0 - 2**-8, 0.1], dtype=np.float32)
    got = wl.bits16_to_f64(wl.f32_to_bits16(f, "bf16"), "bf16")
    assert list(got[:4]) == [1.0, 1.0, 1.0 + 2**-6, -1.0]   # ties go to the even mantissa
    assert abs(got[4] - 0.1) <= 2**-4 * 2**-8


def test_host_pool_matches_block_generator():
    m = wl.Model("t", 2, 2, 2, 8, 4, "f16")
    pool = wl.gen_pool_host(5, wl.STREAM_SRC, m, 6).reshape(m.L, 2, 6, m.H, m.B, m.D)
    for p, b in ((0, 0), (3, 5), (2, 1)):
        assert np.array_equal(pool[p // 2, p % 2, b], wl.gen_block(5, wl.STREAM_SRC, m, p, b))


@pytest.mark.parametrize("name", wl.CONFIG_NAMES)
def test_config_structure(name):
    w = wl.make(name)
    m = w.model
    assert np.array_equal(w.lens, wl.make(name).lens)            # seeded
    used = np.concatenate(w.src_tables)
    assert len(np.unique(used)) == len(used) and used.max() < w.n_blocks_src
    for ln, t in zip(w.lens, w.src_tables):
        assert len(t) == -(-int(ln) // m.B)
    assert (w.k >= 0).all() and (w.k <= w.lens[w.migrate_ids]).all()
    assert int((w.dst_occupied == 0).sum()) >= sum(w.n_dst_blocks())
    if name == "tiny":
        assert len(w.lens) == 8 and len(w.k) == 4 and w.lens.max() <= 256
        assert (w.k == w.lens[:4]).all() and not w.dst_occupied.any()
    if name == "llama2_7b":
        assert len(w.lens) == 64 and len(w.k) == 8 and w.lens.max() <= 4096
        assert w.n_blocks_src == 16384 and m.block_bytes == 8 << 20
    if name == "llama3_8b_gqa":
        assert len(w.lens) == 256 and len(w.k) == 32 and w.lens.max() <= 8192
        assert (w.k == (3 * w.lens[:32]) // 4).all()
        assert 0.48 < w.dst_occupied.mean() < 0.52 and w.n_blocks_dst == 65536
        assert 500 < np.median(w.lens) < 2000
    if name == "llama2_13b_long":
        assert list(w.lens) == [32768] * 4 and 0.28 < w.dst_occupied.mean() < 0.32


def test_shrunken_configs_keep_structure():
    w = wl.make("llama3_8b_gqa", n_blocks_src=512, n_blocks_dst=512, n_requests=12, n_migrate=3,
                len_cap=300)
    assert w.model is wl.LLAMA3_8B and len(w.k) == 3 and w.lens.max() <= 300
    assert np.concatenate(w.src_tables).max() < 512


def test_mixed_scenario_structure():
    from kvm_workload import mixed
    sc = mixed.make()
    assert [m.name for m in sc.models] == ["llama2_7b", "llama3_8b_gqa", "llama2_13b"]
    assert len(sc.requests) == 512 and len(sc.orders) == 200
    assert max(r.length for r in sc.requests) <= 16384
    assert sc.arena_bytes < 260 * 2**30
    for mi, m in enumerate(sc.models):
        for h in range(2):
            ids = np.concatenate([r.table for r in sc.requests if r.model == mi and r.half == h])
            assert len(np.unique(ids)) == len(ids) and ids.max() < sc.half_blocks[mi]
            assert 0.5 < mixed.occupancy(sc, mi, h).mean() < 0.8      # fragmented, not full
            assert sc.half_offset[mi][h] % (2 << 20) == 0
    ends = sorted((sc.half_offset[mi][h], sc.half_offset[mi][h] + sc.half_blocks[mi] * m.block_bytes)
                  for mi, m in enumerate(sc.models) for h in range(2))
    assert all(a[1] <= b[0] for a, b in zip(ends, ends[1:])) and ends[-1][1] <= sc.arena_bytes
    assert all(0.5 <= u <= 1.0 and 0 <= r < 512 for r, u in sc.orders)
    again = mixed.make()
    assert [r.length for r in again.requests] == [r.length for r in sc.requests] and again.orders == sc.orders
