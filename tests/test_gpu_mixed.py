"""Multi-LLM mixed pool: one arena, three KV layouts, a seeded stream of migration
orders run back to back on one stream with a decode check after each.

Shrunken case (three layouts with 2 layers, short requests): the whole arena is
compared bit for bit with the CPU oracle carrying out the same orders, tables
included, and every order's decode output is compared with the fp64 oracle.
Full-size case (243 GiB arena, 512 requests, 200 orders): decode over the
destination equals decode over the source bit for bit for every order, sampled
decode rows match the oracle, every live request's blocks hold the generator's
bytes of the blocks it started in, blocks never handed out are unchanged, and the
free lists equal the complement of the live tables.
"""
import numpy as np
import pytest
import torch

import kvm_workload as wl
import paper_2501_06709_amd as kvm
from kvm_workload import device as wl_device
from kvm_workload import mixed
from paper_2501_06709_amd.migrator import DevicePool, Migrator

from gpu_util import DEV

pytestmark = pytest.mark.gpu
TOL = 2e-3


def build_device(sc):
    arena = torch.empty(sc.arena_bytes, dtype=torch.uint8, device=DEV)
    pools = []
    for mi, m in enumerate(sc.models):
        n = sc.half_blocks[mi]
        lay = kvm.kvm_layout_canonical(m.L, m.H, m.Hq, m.D, m.B, m.dtype, n)
        halves = []
        for h in range(2):
            off = sc.half_offset[mi][h]
            region = arena[off:off + n * m.block_bytes]
            wl_device.fill_pool(region, m, n, sc.seed, sc.stream(mi, h))
            halves.append(DevicePool(region, n, lay, mixed.occupancy(sc, mi, h)))
        pools.append(halves)
    torch.cuda.synchronize()
    return arena, pools


def order_k(rq, u):
    return int(np.floor(u * rq.length))


def test_mixed_pool_shrunken_matches_oracle_everywhere(oracle):
    sc = mixed.make(n_requests=48, n_orders=80, median=40, cap=150, models=mixed.small_models())
    arena, pools = build_device(sc)
    host = arena.cpu().numpy().view(np.uint16).copy()
    # oracle side: own free lists, own tables, host arena
    o_free = [[oracle.FreeList(sc.half_blocks[mi], mixed.occupancy(sc, mi, h)) for h in range(2)]
              for mi in range(len(sc.models))]
    o_tab = [rq.table.copy() for rq in sc.requests]
    o_len = [rq.length for rq in sc.requests]
    o_half = [rq.half for rq in sc.requests]
    max_nb = max(len(rq.table) for rq in sc.requests)
    # depth 1: a source is released before the next order allocates, as the oracle
    # side does, so both allocators see the same free lists
    mig = Migrator(DEV, max_nb, depth=1)
    moved = skipped = 0
    for oi, (ri, u) in enumerate(sc.orders):
        rq = sc.requests[ri]
        m = sc.models[rq.model]
        k = order_k(rq, u)
        src, dst = pools[rq.model][rq.half], pools[rq.model][1 - rq.half]
        q = wl.gen_q(sc.seed + oi, m, 1)
        q_dev = torch.from_numpy(q.view(np.int16)).to(DEV)
        out = torch.zeros(q.shape, dtype=torch.float32, device=DEV)
        mig.drain()
        # oracle
        exp_ids = o_free[rq.model][1 - rq.half].alloc(-(-k // m.B))
        try:
            ids = mig.move(rq.table, rq.length, src, dst, k, decode=(q_dev, out, None, 0))
        except kvm.KvmError as e:
            assert e.status == kvm.KVM_ENOMEM and exp_ids is None
            skipped += 1
            continue
        assert exp_ids is not None and list(ids) == exp_ids
        n = sc.half_blocks[rq.model]
        st = oracle.canonical_strides(m.L, m.H, m.D, m.B, n)
        so, do = sc.half_offset[rq.model][o_half[ri]] // 2, sc.half_offset[rq.model][1 - o_half[ri]] // 2
        span = n * m.block_bytes // 2
        oracle.migrate(host[so:so + span], st, host[do:do + span], st, m.L, m.H, m.D, m.B,
                       [0, len(o_tab[ri])], o_tab[ri], [0, len(exp_ids)], exp_ids, [k])
        if k > 0:
            ref = oracle.paged_decode(host[do:do + span], st, m.L, m.H, m.Hq, m.D, m.B, m.dtype,
                                      [0, len(exp_ids)], exp_ids, [k], q)
            torch.cuda.synchronize()
            err = np.abs(out.cpu().numpy() - ref).max()
            assert err < TOL, (oi, err)
        o_free[rq.model][o_half[ri]].release(o_tab[ri])
        o_tab[ri], o_len[ri], o_half[ri] = np.array(exp_ids, np.int32), k, 1 - o_half[ri]
        rq.table, rq.length, rq.half = ids, k, 1 - rq.half
        moved += 1
    mig.drain()
    torch.cuda.synchronize()
    assert moved >= 60, (moved, skipped)
    assert np.array_equal(arena.cpu().numpy().view(np.uint16), host), "arena differs from the oracle's"
    for mi in range(len(sc.models)):
        for h in range(2):
            assert pools[mi][h].free.available() == o_free[mi][h].available()


def test_staged_orders_share_one_upload(oracle):
    """Orders staged in groups of five (one table upload per group), requests that
    appear twice in a group included: every order's decode over its destination
    matches the fp64 oracle on the request's logical content, every live request
    ends with the bytes it started with, the free lists are the complement of the
    live tables."""
    sc = mixed.make(n_requests=48, n_orders=80, median=40, cap=150, models=mixed.small_models())
    arena, pools = build_device(sc)
    start = arena.cpu().numpy().view(np.uint16).copy()

    def logical(rq, n_tok):
        """[2L][H][n_tok][D] content of the request's first n_tok tokens, from the
        arena as it was before any order, through the blocks the request started in."""
        m = sc.models[rq.model]
        n = sc.half_blocks[rq.model]
        out = np.zeros((2 * m.L, m.H, n_tok, m.D), np.uint16)
        for j in range(-(-n_tok // m.B)):
            oh, ob = rq.origin[j]
            off = sc.half_offset[rq.model][oh] // 2
            planes = start[off:off + n * m.block_bytes // 2].reshape(2 * m.L, n, m.H, m.B, m.D)
            ns = min(m.B, n_tok - j * m.B)
            out[:, :, j * m.B:j * m.B + ns] = planes[:, ob, :, :ns]
        return out

    mig = Migrator(DEV, max(len(rq.table) for rq in sc.requests), depth=4, max_staged=5)
    checks = []
    moved = 0
    for oi, (ri, u) in enumerate(sc.orders):
        rq = sc.requests[ri]
        m = sc.models[rq.model]
        k = order_k(rq, u)
        q = wl.gen_q(sc.seed + oi, m, 1)
        q_dev = torch.from_numpy(q.view(np.int16)).to(DEV)
        out = torch.zeros(q.shape, dtype=torch.float32, device=DEV)
        try:
            ids = mig.stage(rq.table, rq.length, pools[rq.model][rq.half], pools[rq.model][1 - rq.half], k,
                            decode=(q_dev, out, None, 0))
        except kvm.KvmError as e:
            assert e.status == kvm.KVM_ENOMEM
            continue
        if k > 0:
            checks.append((oi, rq, k, q, q_dev, out, logical(rq, k)))   # content now: origin shrinks later
        rq.table, rq.length, rq.half = ids, k, 1 - rq.half
        rq.origin = rq.origin[:len(ids)]
        moved += 1
    mig.drain()
    torch.cuda.synchronize()
    assert moved >= 60
    for oi, rq, k, q, _, out, kv in checks:                   # kv: [2L][H][k][D]
        m = sc.models[rq.model]
        nb = -(-k // m.B)
        pad = np.zeros((2 * m.L, m.H, nb * m.B, m.D), np.uint16)
        pad[:, :, :k] = kv
        # a contiguous one-request pool in the canonical layout [layer][kv][block][head][slot][dim]
        pool = pad.reshape(m.L, 2, m.H, nb, m.B, m.D).transpose(0, 1, 3, 2, 4, 5).copy()
        st = oracle.canonical_strides(m.L, m.H, m.D, m.B, nb)
        ref = oracle.paged_decode(pool.reshape(-1), st, m.L, m.H, m.Hq, m.D, m.B, m.dtype, [0, nb],
                                  np.arange(nb), [k], q)
        err = np.abs(out.cpu().numpy() - ref).max()
        assert err < TOL, (oi, err)
    end = arena.cpu().numpy().view(np.uint16)
    for rq in sc.requests:
        if rq.length == 0:
            continue
        m = sc.models[rq.model]
        n = sc.half_blocks[rq.model]
        off = sc.half_offset[rq.model][rq.half] // 2
        planes = end[off:off + n * m.block_bytes // 2].reshape(2 * m.L, n, m.H, m.B, m.D)
        exp = logical(rq, rq.length)
        for j in range(-(-rq.length // m.B)):
            ns = min(m.B, rq.length - j * m.B)
            assert np.array_equal(planes[:, int(rq.table[j]), :, :ns], exp[:, :, j * m.B:j * m.B + ns])
    for mi in range(len(sc.models)):
        for h in range(2):
            live = sum(len(rq.table) for rq in sc.requests if rq.model == mi and rq.half == h)
            assert pools[mi][h].free.available() == sc.half_blocks[mi] - live


def region_checksums(arena, sc):
    out = {}
    for mi, m in enumerate(sc.models):
        n = sc.half_blocks[mi]
        for h in range(2):
            off = sc.half_offset[mi][h]
            out[(mi, h)] = wl_device.plane_block_checksums(arena[off:off + n * m.block_bytes], m, n)
    return out


def test_mixed_pool_full_size(oracle):
    sc = mixed.make()
    free_b, _ = torch.cuda.mem_get_info()
    if sc.arena_bytes + (12 << 30) > free_b:
        pytest.skip("needs %.0f GiB of HBM" % (sc.arena_bytes / 2**30))
    arena, pools = build_device(sc)
    before = region_checksums(arena, sc)
    handed_out = {key: np.zeros(sc.half_blocks[key[0]], bool) for key in before}
    rng = np.random.default_rng(3)
    max_nb = max(len(rq.table) for rq in sc.requests)
    mig = Migrator(DEV, max_nb)
    moved = skipped = 0
    worst = 0.0
    for oi, (ri, u) in enumerate(sc.orders):
        rq = sc.requests[ri]
        m = sc.models[rq.model]
        k = order_k(rq, u)
        src, dst = pools[rq.model][rq.half], pools[rq.model][1 - rq.half]
        q = wl.gen_q(sc.seed + oi, m, 1)
        q_dev = torch.from_numpy(q.view(np.int16)).to(DEV)
        out = torch.zeros(q.shape, dtype=torch.float32, device=DEV)
        out_src = torch.zeros_like(out)
        # decode over the first k tokens of the source, before anything moves
        if k > 0:
            tab_dev = torch.from_numpy(np.asarray(rq.table, np.int32)).to(DEV)
            sb = kvm.Batch([0, len(rq.table)], rq.table, [k], tab_dev)
            kvm.kvm_paged_decode(src.pool, sb, q_dev, out_src)
        try:
            ids = mig.move(rq.table, rq.length, src, dst, k, decode=(q_dev, out, None, 0))
        except kvm.KvmError as e:
            assert e.status == kvm.KVM_ENOMEM
            skipped += 1
            continue
        handed_out[(rq.model, 1 - rq.half)][ids] = True
        torch.cuda.synchronize()
        assert torch.equal(out, out_src), "order %d: decode over destination != decode over source" % oi
        if k > 0:
            # one sampled (layer, query head) row against the fp64 oracle on regenerated K/V
            l, hq = int(rng.integers(m.L)), int(rng.integers(m.Hq))
            g = hq // (m.Hq // m.H)
            nb = -(-k // m.B)
            wsel = (g * m.B * m.D + np.arange(m.B * m.D)).astype(np.uint32)
            kv = np.zeros((2, nb, m.B * m.D), dtype=np.uint16)
            for j in range(nb):
                oh, ob = rq.origin[j]
                for c in range(2):
                    kv[c, j] = wl.gen_values(sc.seed, sc.stream(rq.model, oh), 2 * l + c, ob, wsel, m.dtype)
            st1 = oracle.canonical_strides(1, 1, m.D, m.B, nb)
            ref = oracle.paged_decode(kv.reshape(-1), st1, 1, 1, 1, m.D, m.B, m.dtype, [0, nb],
                                      np.arange(nb), [k], q[0, l, hq].reshape(1, 1, 1, m.D))
            err = float(np.abs(out[0, l, hq].cpu().numpy().astype(np.float64) - ref[0, 0, 0]).max())
            worst = max(worst, err)
            assert err < TOL, (oi, err)
        rq.table, rq.length, rq.half = ids, k, 1 - rq.half
        rq.origin = rq.origin[:len(ids)]
        moved += 1
    mig.drain()
    torch.cuda.synchronize()
    assert moved >= 150, (moved, skipped)
    # blocks never handed out are unchanged; free lists = complement of the live tables
    after = region_checksums(arena, sc)
    for key in before:
        changed = (after[key] != before[key]).any(dim=0).cpu().numpy()
        assert not (changed & ~handed_out[key]).any(), "a block that was never allocated changed"
        mi, h = key
        live = int(mixed.occupancy(sc, mi, h).sum())
        assert pools[mi][h].free.available() == sc.half_blocks[mi] - live
    # content identity: sampled live blocks hold the bytes of the blocks they started in
    movers = [rq for rq in sc.requests if rq.length > 0 and rq.origin and
              (rq.half, int(rq.table[0])) != rq.origin[0]]
    for rq in [movers[i] for i in rng.choice(len(movers), size=12)]:
        m = sc.models[rq.model]
        n = sc.half_blocks[rq.model]
        off = sc.half_offset[rq.model][rq.half]
        run = m.H * m.B * m.D
        planes = arena[off:off + n * m.block_bytes].view(torch.int16).view(2 * m.L, n, run)
        nb = -(-rq.length // m.B)
        for j in {0, nb - 1, int(rng.integers(nb))}:
            p = int(rng.integers(2 * m.L))
            ns = min(m.B, rq.length - j * m.B)
            oh, ob = rq.origin[j]
            exp = wl.gen_block(sc.seed, sc.stream(rq.model, oh), m, p, ob)
            got = planes[p, int(rq.table[j])].cpu().numpy().view(np.uint16).reshape(m.H, m.B, m.D)
            assert np.array_equal(got[:, :ns], exp[:, :ns])
    print("mixed: %d orders moved, %d skipped for lack of blocks, worst sampled decode error %.2e"
          % (moved, skipped, worst))
