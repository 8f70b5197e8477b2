"""End to end: the scheduler-generated order stream drives the migration path.

Per time slot: completed requests release their blocks; the slot's net move list
goes through the hybrid-migration divider (one shared link with a communication
boundary, a computation boundary per destination GPU); KV-class moves run through
kvm_migrate into blocks popped from the destination GPU's free list, token-class
moves arrive with k = 0 (their cache is to be recomputed, so their content is no
longer tracked), deferred moves are retried as KV moves at the end of the slot;
arrivals get blocks and generator-filled KV.  The CPU oracle carries out the same
stream on a host arena with its own allocator and divider; tables, classes and the
whole arena must agree bit for bit at the end.
"""
import numpy as np
import pytest
import torch

import kvm_workload as wl
import paper_2501_06709_amd as kvm
from kvm_workload import scheduler as sc
from paper_2501_06709_amd.migrator import DevicePool

from gpu_util import DEV

pytestmark = pytest.mark.gpu

M = wl.Model("sched", 2, 4, 8, 128, 16, "bf16")
CAP_BLOCKS = 256                      # KV capacity of one simulated GPU, in blocks
POOL_BLOCKS = 352                     # physical blocks per pool: headroom for copy-then-release


def test_scheduler_stream_through_divider_and_migrate(oracle):
    C = CAP_BLOCKS * M.block_bytes
    # the simulator's "token" is one block here, so sizes are exact block counts
    tr = sc.simulate(C, M.block_bytes, n_slots=120, arrival_rate=2.0, median=40, sigma=0.9,
                     cap_tokens=CAP_BLOCKS, growth_tokens=1, static_sizes=True, seed=21)
    n_pools = tr.peak_gpus + 2
    lay = kvm.kvm_layout_canonical(M.L, M.H, M.Hq, M.D, M.B, M.dtype, POOL_BLOCKS)
    pool_bytes = POOL_BLOCKS * M.block_bytes
    arena = torch.zeros(n_pools * pool_bytes, dtype=torch.uint8, device=DEV)
    host = np.zeros(n_pools * pool_bytes // 2, dtype=np.uint16)
    pools = [DevicePool(arena[i * pool_bytes:(i + 1) * pool_bytes], POOL_BLOCKS, lay) for i in range(n_pools)]
    o_free = [oracle.FreeList(POOL_BLOCKS) for _ in range(n_pools)]
    st = oracle.canonical_strides(M.L, M.H, M.D, M.B, POOL_BLOCKS)
    span = pool_bytes // 2
    slot_of, load = {}, {}            # simulated gpu id -> pool index, live requests per gpu id
    table, tracked = {}, {}           # request -> (gpu id, ids); request -> content still meaningful
    origin = {}                       # request -> block ids it was prefilled into
    n_kv = n_tok = n_def = 0

    def pool_index(gid):
        if gid not in slot_of:
            used = set(slot_of.values())
            slot_of[gid] = min(i for i in range(n_pools) if i not in used)
            load[gid] = 0
        return slot_of[gid]

    def leave(gid):
        load[gid] -= 1
        if load[gid] == 0:
            del slot_of[gid], load[gid]

    for slot in range(len(tr.orders)):
        for rid in tr.departures[slot]:
            gid, ids = table.pop(rid)
            tracked.pop(rid)
            pools[slot_of[gid]].free.free(ids)
            o_free[slot_of[gid]].release(ids)
            leave(gid)
        orders = tr.orders[slot]
        if orders:
            total = sum(o[3] for o in orders)
            moves = [(0, dst, nbytes, nbytes // M.bytes_per_token) for _, _, dst, nbytes in orders]
            gids = sorted({o[2] for o in orders})
            remap = {g: i for i, g in enumerate(gids)}
            moves = [(0, remap[d], b, t) for _, d, b, t in moves]
            comm, comp = [int(0.6 * total)], [CAP_BLOCKS * M.B // 4] * len(gids)
            cls = kvm.kvm_divide_moves(moves, comm, comp, kvm.KVM_BEST_FIT)
            assert list(cls) == oracle.divide_moves(moves, comm, comp, "best_fit")
            # deferred moves run as KV moves after the others
            order_ix = sorted(range(len(orders)), key=lambda i: cls[i] == kvm.KVM_CLASS_DEFER)
            for i in order_ix:
                rid, src_gid, dst_gid, nbytes = orders[i]
                _, ids = table[rid]
                tokens = nbytes // M.bytes_per_token
                k = 0 if cls[i] == kvm.KVM_CLASS_TOKENS else tokens
                n_kv += cls[i] == kvm.KVM_CLASS_KV
                n_tok += cls[i] == kvm.KVM_CLASS_TOKENS
                n_def += cls[i] == kvm.KVM_CLASS_DEFER
                sp, dp = slot_of[src_gid], pool_index(dst_gid)
                load[dst_gid] += 1
                nb = len(ids)                       # the request keeps its blocks' worth of room
                new_ids = pools[dp].free.alloc(nb)
                exp_ids = o_free[dp].alloc(nb)
                assert list(new_ids) == exp_ids
                if k > 0:
                    dev_s = torch.from_numpy(np.asarray(ids, np.int32)).to(DEV)
                    dev_d = torch.from_numpy(new_ids).to(DEV)
                    sb = kvm.Batch([0, nb], ids, [k], dev_s)
                    db = kvm.Batch([0, nb], new_ids, [k], dev_d)
                    kvm.kvm_migrate(pools[sp].pool, sb, pools[dp].pool, db)
                    torch.cuda.synchronize()
                    oracle.migrate(host[sp * span:(sp + 1) * span], st, host[dp * span:(dp + 1) * span], st,
                                   M.L, M.H, M.D, M.B, [0, nb], ids, [0, nb], exp_ids, [k])
                else:
                    tracked[rid] = False
                pools[sp].free.free(ids)
                o_free[sp].release(ids)
                leave(src_gid)
                table[rid] = (dst_gid, new_ids)
        for rid, gid, nbytes in tr.arrivals[slot]:
            p = pool_index(gid)
            load[gid] += 1
            nb = nbytes // M.block_bytes
            ids = pools[p].free.alloc(nb)
            assert list(ids) == o_free[p].alloc(nb)
            # "prefill": the request's KV appears in its blocks (generator stream = request id)
            for b in ids:
                blk = np.stack([wl.gen_block(7, 100 + rid, M, pl, int(b)) for pl in range(2 * M.L)])
                view = host[p * span:(p + 1) * span].reshape(2 * M.L, POOL_BLOCKS, -1)
                view[:, b] = blk.reshape(2 * M.L, -1)
                dview = arena[p * pool_bytes:(p + 1) * pool_bytes].view(torch.int16).view(2 * M.L, POOL_BLOCKS, -1)
                dview[:, int(b)] = torch.from_numpy(blk.reshape(2 * M.L, -1).view(np.int16)).to(DEV)
            table[rid] = (gid, ids)
            origin[rid] = [int(b) for b in ids]
            tracked[rid] = True
    torch.cuda.synchronize()
    assert n_kv >= 15 and n_tok >= 5 and n_def >= 1, (n_kv, n_tok, n_def)
    assert np.array_equal(arena.cpu().numpy().view(np.uint16), host), "arena differs from the oracle's"
    for i in range(n_pools):
        assert pools[i].free.available() == o_free[i].available()
    # every request whose cache only ever travelled as KV still holds, block by block in
    # logical order, the bytes it was prefilled with (content identity travels with it)
    checked = 0
    for rid, (gid, ids) in table.items():
        if not tracked[rid] or checked >= 12:
            continue
        p = slot_of[gid]
        view = arena[p * pool_bytes:(p + 1) * pool_bytes].view(torch.int16).view(2 * M.L, POOL_BLOCKS, -1)
        for j in {0, len(ids) - 1}:
            pl = (rid + j) % (2 * M.L)
            got = view[pl, int(ids[j])].cpu().numpy().view(np.uint16)
            assert np.array_equal(got, wl.gen_block(7, 100 + rid, M, pl, origin[rid][j]).reshape(-1))
        checked += 1
    assert checked > 5
    print("stream: %d KV moves, %d token moves, %d deferred, %d simulated GPUs at peak"
          % (n_kv, n_tok, n_def, tr.peak_gpus))
