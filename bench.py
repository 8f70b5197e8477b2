#!/usr/bin/env python3
"""Benchmark of the paged-KV migration hot path on one MI355X.

A step is one pass of the whole path over the batch of requests to migrate:
  1. destination blocks popped from the destination free list, new block table
     uploaded;
  2. kvm_pack   (gather into the staging buffer)
  3. kvm_unpack (scatter the staging buffer into the destination blocks)
  4. kvm_migrate (the same move fused, no staging; same destination tables)
  5. kvm_paged_decode over the destination cache
  6. source blocks returned to the source free list once the copies are done
followed by the bookkeeping that lets the next step start from the same state
(source ids reserved again, destination ids freed).  All of it is inside the
timed region.

`value` = bytes read + written by pack, unpack and fused migrate (6 x payload per
step) divided by the whole step time (decode check and host steps are in the
time, not in the bytes), in GB/s.  `roofline` is the fused migrate kernel alone:
2 x payload / its average duration measured with HIP events on the launch
stream inside the timed region.  `cpu_baseline` times the CPU oracle on a stated
sample of the same workload, same byte accounting.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0

# HBM bytes per fused-migrate launch, measured with rocprofv3 --pmc (a FETCH_SIZE
# run and a WRITE_SIZE run, each scaled by what the same counter reads for the
# plain copy kernel of known size in the same run); the counter summaries are in
# profiles/kvm_migrate_llama3_8b_gqa_pmc_hbm.md.  Workloads without a measurement
# report null.
MEASURED_TRAFFIC_BYTES = {"llama3_8b_gqa": 7995046550}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="llama3_8b_gqa")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=16, help="requests in the oracle's sample")
    ap.add_argument("--unroll", type=int, default=None)
    ap.add_argument("--nontemporal", type=int, default=None)
    ap.add_argument("--order", type=int, default=None)
    ap.add_argument("--split-target", type=int, default=None)
    ap.add_argument("--no-verify", action="store_true")
    ap.add_argument("--q-heads", type=int, default=None,
                    help="query heads of the decode leg (a multiple of the KV heads); e.g. 64 on "
                         "llama3_8b_gqa gives the 70B-class group of eight over the same KV")
    return ap.parse_args()


def fit_pools(w, free_bytes, extra_bytes, log):
    """Shrink the pools (never the requests) when 2 pools + staging exceed HBM."""
    m = w.model
    need = (w.n_blocks_src + w.n_blocks_dst) * m.block_bytes + extra_bytes
    budget = free_bytes - (3 << 30)
    if need <= budget:
        return w
    import kvm_workload as wl
    scale = (budget - extra_bytes) / ((w.n_blocks_src + w.n_blocks_dst) * m.block_bytes)
    nbs, nbd = int(w.n_blocks_src * scale), int(w.n_blocks_dst * scale)
    log("pools shrunk to fit HBM: src %d -> %d blocks, dst %d -> %d blocks"
        % (w.n_blocks_src, nbs, w.n_blocks_dst, nbd))
    w2 = wl.make(w.name, n_blocks_src=nbs, n_blocks_dst=nbd)
    w2.notes.append("pools shrunk to fit HBM: src %d, dst %d blocks" % (nbs, nbd))
    return w2


def cpu_baseline(w, src_mem, staging_bytes_per_token, n_sample, log):
    """Time the oracle (pack, unpack, migrate, decode) on the first n_sample
    migrated requests, on a compact host pool holding only their blocks."""
    import concurrent.futures as cf

    import numpy as np
    import torch

    import kvm_workload as wl
    from oracle import oracle as orc

    m = w.model
    n_sample = min(n_sample, len(w.k))
    ks = w.k[:n_sample]
    tabs = [w.src_tables[i] for i in w.migrate_ids[:n_sample]]
    nbk = [-(-int(k) // m.B) for k in ks]
    used = np.concatenate([t[:n] for t, n in zip(tabs, nbk)]).astype(np.int64)
    n_loc = len(used)
    # compact host source pool: the sampled blocks, in a seeded shuffled order
    rng = np.random.default_rng(w.seed)
    order = rng.permutation(n_loc).astype(np.int32)     # local id of the i-th used block
    run = m.H * m.B * m.D
    planes = src_mem.view(torch.int16).view(2 * m.L, w.n_blocks_src, run)
    host_src = np.empty((2 * m.L, n_loc, run), dtype=np.uint16)
    idx = torch.from_numpy(used).to(src_mem.device)
    inv = np.empty(n_loc, dtype=np.int64)
    inv[order] = np.arange(n_loc)
    for p in range(2 * m.L):
        host_src[p, order] = planes[p].index_select(0, idx).cpu().numpy().view(np.uint16)
    host_src = host_src.reshape(-1)
    host_dst = np.zeros_like(host_src)
    st = orc.canonical_strides(m.L, m.H, m.D, m.B, n_loc)
    s_tabs, p = [], 0
    for n in nbk:
        s_tabs.append(order[p:p + n].copy())
        p += n
    d_ids = orc.FreeList(n_loc).alloc(n_loc)
    d_tabs, p = [], 0
    for n in nbk:
        d_tabs.append(np.array(d_ids[p:p + n], dtype=np.int32))
        p += n
    q = wl.gen_q(w.seed, m, n_sample)
    threads = min(16, os.cpu_count() or 1)
    payload = int(ks.astype(np.int64).sum()) * m.bytes_per_token
    stage = [np.zeros(orc.staging_elems(m.L, m.H, m.D, [k]), dtype=np.uint16) for k in ks]

    def one(r):
        return [0, len(s_tabs[r])], s_tabs[r], [0, len(d_tabs[r])], d_tabs[r], [int(ks[r])]

    def copy_unit(args):
        r, l = args
        so, sb, do, db, k = one(r)
        orc.pack(host_src, st, m.L, m.H, m.D, m.B, so, sb, k, stage=stage[r], layers=(l, l + 1))
        orc.unpack(stage[r], host_dst, st, m.L, m.H, m.D, m.B, do, db, k, layers=(l, l + 1))
        orc.migrate(host_src, st, host_dst, st, m.L, m.H, m.D, m.B, so, sb, do, db, k,
                    layers=(l, l + 1))

    def decode_unit(r):
        so, sb, do, db, k = one(r)
        return orc.paged_decode(host_dst, st, m.L, m.H, m.Hq, m.D, m.B, m.dtype, do, db, k,
                                q[r:r + 1])

    t0 = time.perf_counter()
    with cf.ThreadPoolExecutor(threads) as ex:
        list(ex.map(copy_unit, [(r, l) for r in range(n_sample) for l in range(m.L)]))
        t1 = time.perf_counter()
        list(ex.map(decode_unit, range(n_sample)))
    t2 = time.perf_counter()
    log("cpu oracle: %d requests, payload %.1f MiB, copies %.2f s, decode %.2f s on %d threads"
        % (n_sample, payload / 2**20, t1 - t0, t2 - t1, threads))
    return {"value": round(6 * payload / (t2 - t0) / 1e9, 4), "unit": "GB/s", "cores": threads,
            "kind": "oracle",
            "sample": "first %d of %d migrated requests (%d tokens, %.1f MiB payload); pack+unpack+"
                      "migrate over (request, layer) units, fp64 decode over requests; copies %.2f s,"
                      " decode %.2f s" % (n_sample, len(w.k), int(ks.sum()), payload / 2**20,
                                          t1 - t0, t2 - t1)}


def bench_mixed(a, log):
    """Multi-LLM mixed pool: the seeded order stream run back to back on one stream
    (allocation, one table upload per 16 orders, one fused migrate and one decode
    launch per (model, direction) of those 16, deferred source release), host overhead
    included.  One step = one order."""
    import numpy as np
    import torch

    import kvm_workload as wl
    import paper_2501_06709_amd as kvm
    from kvm_workload import device as wl_device
    from kvm_workload import mixed
    from paper_2501_06709_amd.migrator import DevicePool, Migrator

    dev = torch.device("cuda:0")
    sc = mixed.make()
    arena = torch.empty(sc.arena_bytes, dtype=torch.uint8, device=dev)
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
    n_stage = 16
    qs = [torch.from_numpy(wl.gen_q(sc.seed, m, n_stage).view(np.int16)).to(dev) for m in sc.models]
    outs = [torch.zeros(q.shape, dtype=torch.float32, device=dev) for q in qs]
    ws = torch.empty(32 << 20, dtype=torch.uint8, device=dev)      # decode split workspace
    torch.cuda.synchronize()
    log("mixed arena %.1f GiB, %d requests, %d orders" % (sc.arena_bytes / 2**30, len(sc.requests),
                                                          len(sc.orders)))
    mig = Migrator(dev, max(len(r.table) for r in sc.requests), max_staged=n_stage, decode_workspace=ws,
                   time_copies=True)
    # warm-up, untimed: one block of every model moved into a free block of its other
    # half and one decode over it, so that the first timed order does not pay for
    # loading the kernels; the block is handed back, no request's table changes
    for mi, m in enumerate(sc.models):
        rq = next(r for r in sc.requests if r.model == mi)
        got = mig.move(rq.table[:1], min(rq.length, m.B), pools[mi][rq.half], pools[mi][1 - rq.half],
                       min(rq.length, m.B), decode=(qs[mi], outs[mi], 0))
        mig.drain()                                   # would release the source block ...
        pools[mi][rq.half].free.reserve(rq.table[:1])  # ... which stays in use
        pools[mi][1 - rq.half].free.free(got)
    torch.cuda.synchronize()
    mig.copy_marks.clear()
    launches0 = mig.launches
    moved = skipped = blocks = 0
    nbytes = 0
    t0 = time.perf_counter()
    for ri, u in sc.orders:
        rq = sc.requests[ri]
        m = sc.models[rq.model]
        k = int(np.floor(u * rq.length))
        try:
            # staged: up to 16 orders per flush; a flush is one table upload and, per
            # (model, direction), one fused-migrate and one decode launch over its orders
            ids = mig.stage(rq.table, rq.length, pools[rq.model][rq.half], pools[rq.model][1 - rq.half],
                            k, decode=(qs[rq.model], outs[rq.model], len(mig.staged) % n_stage))
        except kvm.KvmError:
            skipped += 1
            continue
        rq.table, rq.length, rq.half = ids, k, 1 - rq.half
        moved += 1
        blocks += len(ids)
        nbytes += 2 * k * m.bytes_per_token
    t_host = time.perf_counter() - t0
    mig.drain()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    log("host loop %.1f ms" % (t_host * 1e3))
    log("%d orders moved (%d skipped) in %.1f ms, %d library calls" % (moved, skipped, dt * 1e3,
                                                                      mig.launches - launches0))
    gbs = nbytes / dt / 1e9
    copy_ms = sum(e0.elapsed_time(e1) for e0, e1, _ in mig.copy_marks)
    copy_bytes = sum(b for _, _, b in mig.copy_marks)
    copy_gbs = copy_bytes / (copy_ms * 1e-3) / 1e9
    log("fused migrate launches: %d, %.2f ms in total, %.0f GB/s" % (len(mig.copy_marks), copy_ms, copy_gbs))
    print(json.dumps({
        "metric": "KV migrate GB/s (read+write)", "value": round(gbs, 2), "unit": "GB/s", "n_gpus": 1,
        "steps": moved, "warmup": len(sc.models), "ms_per_step": round(dt * 1e3 / max(moved, 1), 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u16",
        "data": "synthetic",
        "config": {"workload": "mixed", "arena_bytes": sc.arena_bytes, "requests": len(sc.requests),
                   "orders": len(sc.orders), "orders_skipped_no_blocks": skipped,
                   "orders_per_flush": n_stage, "library_calls": mig.launches - launches0,
                   "value_is": "2 x moved bytes per second of wall time over the whole order stream, "
                               "decode over each destination and host work included"},
        "frac_of_hbm_peak": round(gbs / HBM_PEAK_GBS, 4),
        "orders_per_s": round(moved / dt, 1), "migrated_blocks_per_s": round(blocks / dt, 1),
        "roofline": {"kernel": "copy_kernel<migrate> (kvm_migrate), all launches of the stream",
                     "bound": "hbm", "achieved": round(copy_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(copy_gbs / HBM_PEAK_GBS, 4),
                     "launches": len(mig.copy_marks), "algorithmic_bytes": copy_bytes,
                     "traffic": None}}), flush=True)


if __name__ == "__main__":
    main()
