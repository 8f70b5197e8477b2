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
# profiles/kvm_migrate_llama3_8b_gqa_pmc_hbm.md.  A figure is only reported for the
# payload it was measured on (the workloads are seeded, so the payload identifies
# the launch); other workloads, or a changed workload, report null.
MEASURED_TRAFFIC = {"llama3_8b_gqa": {"payload_bytes": 3994157056, "hbm_bytes": 7994907668}}


def measured_traffic(name, payload):
    rec = MEASURED_TRAFFIC.get(name)
    return rec["hbm_bytes"] if rec and rec["payload_bytes"] == payload else None


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--config", default="llama3_8b_gqa")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=32, help="requests in the oracle's sample")
    ap.add_argument("--nontemporal", type=int, default=None)
    ap.add_argument("--order", type=int, default=None)
    ap.add_argument("--split-target", type=int, default=None)
    ap.add_argument("--no-verify", action="store_true")
    ap.add_argument("--no-reference-legs", action="store_true",
                    help="skip the table-free reference access patterns (they overwrite the destination pool)")
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
    # one thread per host core, but never more than the 16 cores a one-GPU machine grants
    host_cores = os.cpu_count() or 1
    threads = min(16, host_cores)
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
    # single thread: the copies of the first two sampled requests, the decode of the shortest one
    n1 = min(2, n_sample)
    p1 = int(ks[:n1].astype(np.int64).sum()) * m.bytes_per_token
    t3 = time.perf_counter()
    for r in range(n1):
        for l in range(m.L):
            copy_unit((r, l))
    t4 = time.perf_counter()
    r_short = int(np.argmin(ks))
    decode_unit(r_short)
    t5 = time.perf_counter()
    pd1 = int(ks[r_short]) * m.bytes_per_token
    log("cpu oracle: %d requests, payload %.1f MiB, copies %.2f s, decode %.2f s on %d threads; one thread: "
        "copies of %d requests %.2f s, decode of one request %.2f s"
        % (n_sample, payload / 2**20, t1 - t0, t2 - t1, threads, n1, t4 - t3, t5 - t4))
    return {"value": round(6 * payload / (t2 - t0) / 1e9, 4), "unit": "GB/s", "cores": threads,
            "kind": "oracle", "host_cpu_count": host_cores,
            "copy_GBs": round(6 * payload / (t1 - t0) / 1e9, 3),
            "decode_GBs": round(payload / (t2 - t1) / 1e9, 4),
            "single_thread": {"copy_GBs": round(6 * p1 / (t4 - t3) / 1e9, 3),
                              "decode_GBs": round(pd1 / (t5 - t4) / 1e9, 5)},
            "sample": "first %d of %d migrated requests (%d tokens, %.1f MiB payload); value: bytes read+"
                      "written by pack, unpack and migrate (6 x payload) over copies + fp64 decode time, "
                      "as the GPU value; copy_GBs: the three copies alone over (request, layer) units; "
                      "decode_GBs: KV bytes read by the fp64 decode; copies %.2f s, decode %.2f s; "
                      "single_thread: copies of the first %d requests, decode of the shortest one"
                      % (n_sample, len(w.k), int(ks.sum()), payload / 2**20, t1 - t0, t2 - t1, n1)}


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
    mig.reset_copy_stats()
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
            # rows: any n_stage consecutive orders (a flush never holds more) get distinct ones
            ids = mig.stage(rq.table, rq.length, pools[rq.model][rq.half], pools[rq.model][1 - rq.half],
                            k, decode=(qs[rq.model], outs[rq.model], (moved + skipped) % n_stage))
        except kvm.KvmError as e:
            if e.status != kvm.KVM_ENOMEM:
                raise
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
    hbm_gbs = 1.5 * nbytes / dt / 1e9      # + the decode's read of every moved byte
    copy_ms, copy_bytes, n_copies = mig.copy_stats()
    copy_gbs = copy_bytes / (copy_ms * 1e-3) / 1e9
    log("fused migrate launches: %d, %.2f ms in total, %.0f GB/s" % (n_copies, copy_ms, copy_gbs))
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
        "sustained_hbm": {"GB/s": round(hbm_gbs, 1), "frac_of_hbm_peak": round(hbm_gbs / HBM_PEAK_GBS, 4),
                          "is": "bytes read + written by the copies plus bytes read by the decodes, per "
                                "second of wall time"},
        "orders_per_s": round(moved / dt, 1), "migrated_blocks_per_s": round(blocks / dt, 1),
        "roofline": {"kernel": "copy_kernel<migrate> (kvm_migrate), all launches of the stream",
                     "bound": "hbm", "achieved": round(copy_gbs, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round(copy_gbs / HBM_PEAK_GBS, 4),
                     "launches": n_copies, "algorithmic_bytes": copy_bytes,
                     "traffic": None}}), flush=True)


def main():
    a = parse()
    if a.gpus != 1:
        print("bench.py measures one GPU: the migration path here has no multi-GPU part "
              "(--gpus %d refused)" % a.gpus, file=sys.stderr)
        sys.exit(2)

    def log(msg):
        print("[bench] " + msg, file=sys.stderr, flush=True)

    import numpy as np
    import torch

    import kvm_workload as wl
    import paper_2501_06709_amd as kvm
    from kvm_workload import device as wl_device

    kvm.lib()  # fails loudly if the HIP library is not built
    for name, val in (("copy.nontemporal", a.nontemporal),
                      ("copy.order", a.order), ("decode.split_target", a.split_target)):
        if val is not None:
            kvm.kvm_set_option(name, val)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    if a.config == "mixed":
        return bench_mixed(a, log)
    w = wl.make(a.config)
    m = w.model
    payload = w.payload_bytes()
    free_b, total_b = torch.cuda.mem_get_info()
    log("HBM free %.1f GiB of %.1f GiB; workload %s payload %.2f GiB"
        % (free_b / 2**30, total_b / 2**30, w.name, payload / 2**30))
    # room beside the pools: staging for at least the largest request, tables, q, out
    w = fit_pools(w, free_b, int(w.k.max()) * m.bytes_per_token + (2 << 30), log)
    if a.q_heads is not None:   # only the decode leg sees the query heads
        import dataclasses
        w.model = m = dataclasses.replace(w.model, Hq=a.q_heads)
        w.notes = list(w.notes) + ["query heads overridden to %d" % a.q_heads]
    payload = w.payload_bytes()

    lay_s = kvm.kvm_layout_canonical(m.L, m.H, m.Hq, m.D, m.B, m.dtype, w.n_blocks_src)
    lay_d = kvm.kvm_layout_canonical(m.L, m.H, m.Hq, m.D, m.B, m.dtype, w.n_blocks_dst)
    src_mem = torch.empty(kvm.kvm_pool_span_bytes(lay_s, w.n_blocks_src), dtype=torch.uint8, device=dev)
    dst_mem = torch.empty(kvm.kvm_pool_span_bytes(lay_d, w.n_blocks_dst), dtype=torch.uint8, device=dev)
    t0 = time.perf_counter()
    wl_device.fill_pool(src_mem, m, w.n_blocks_src, w.seed, wl.STREAM_SRC)
    wl_device.fill_pool(dst_mem, m, w.n_blocks_dst, w.seed, wl.STREAM_DST)
    torch.cuda.synchronize()
    log("pools: src %d blocks (%.1f GiB), dst %d blocks (%.1f GiB), filled in %.2f s"
        % (w.n_blocks_src, src_mem.numel() / 2**30, w.n_blocks_dst, dst_mem.numel() / 2**30,
           time.perf_counter() - t0))
    src_pool = kvm.Pool(src_mem, w.n_blocks_src, lay_s)
    dst_pool = kvm.Pool(dst_mem, w.n_blocks_dst, lay_d)

    # source side: tables of the migrated requests; free list = blocks no live request holds
    s_off, s_blk = w.src_csr()
    s_blk_dev = torch.from_numpy(s_blk).to(dev)
    src_batch = kvm.Batch(s_off, s_blk, w.k, s_blk_dev)
    src_occ = np.zeros(w.n_blocks_src, np.uint8)
    src_occ[np.concatenate(w.src_tables)] = 1
    src_fl = kvm.FreeList(w.n_blocks_src, src_occ)
    dst_fl = kvm.FreeList(w.n_blocks_dst, w.dst_occupied)

    nbk = w.n_dst_blocks()
    n_dst = int(sum(nbk))
    d_off = np.zeros(len(nbk) + 1, np.int32)
    d_off[1:] = np.cumsum(nbk)
    d_blk_pin = torch.empty(max(n_dst, 1), dtype=torch.int32, pin_memory=True)
    d_blk_dev = torch.empty(max(n_dst, 1), dtype=torch.int32, device=dev)
    # The staged path needs a staging buffer; when the whole batch's does not fit
    # beside the pools it is run in groups of consecutive requests.
    free_now, _ = torch.cuda.mem_get_info()
    stage_budget = max(free_now - (4 << 30), 1 << 20)
    groups, g0, acc = [], 0, 0
    for r, kr in enumerate(w.k):
        b = int(kr) * m.bytes_per_token
        if b > stage_budget:
            raise SystemExit("one request's staging (%d B) does not fit in HBM" % b)
        if acc + b > stage_budget:
            groups.append((g0, r))
            g0, acc = r, 0
        acc += b
    groups.append((g0, len(w.k)))
    stage_bytes = max(int(w.k[lo:hi].astype(np.int64).sum()) * m.bytes_per_token for lo, hi in groups)
    staging = torch.empty(max(stage_bytes, 16), dtype=torch.uint8, device=dev)
    if len(groups) > 1:
        log("staged path runs in %d request groups (staging buffer %.1f GiB)"
            % (len(groups), stage_bytes / 2**30))
    q_host = wl.gen_q(w.seed, m, len(w.k))
    q_dev = torch.from_numpy(q_host.view(np.int16)).to(dev)
    out = torch.zeros(q_host.shape, dtype=torch.float32, device=dev)
    probe = kvm.Batch(d_off, np.zeros(n_dst, np.int32), w.k, d_blk_dev)
    ws_bytes = kvm.kvm_decode_workspace_bytes(lay_d, probe)
    ws = torch.empty(max(ws_bytes, 16), dtype=torch.uint8, device=dev)

    def sub_batch(off, blk, blk_dev, lo, hi):
        """Requests [lo,hi) of a batch as a batch of their own (pointer arithmetic only)."""
        o = off[lo:hi + 1] - off[lo]
        return kvm.Batch(o, blk[off[lo]:off[hi]], w.k[lo:hi], blk_dev.data_ptr() + 4 * int(off[lo]))

    src_groups = [sub_batch(s_off, s_blk, s_blk_dev, lo, hi) for lo, hi in groups]
    names = ("pack", "unpack", "migrate", "decode")
    stream = torch.cuda.current_stream()

    def step(events):
        # allocate destination blocks, rewrite and upload the block table
        ids = dst_fl.alloc(n_dst)
        d_blk_pin.numpy()[:n_dst] = ids
        d_blk_dev.copy_(d_blk_pin, non_blocking=True)
        dst_batch = kvm.Batch(d_off, ids, w.k, d_blk_dev)
        marks = []

        def timed(name, fn):
            if events is None:
                return fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            fn()
            e1.record(stream)
            marks.append((name, e0, e1))

        for (lo, hi), sg in zip(groups, src_groups):
            dg = dst_batch if len(groups) == 1 else sub_batch(d_off, ids, d_blk_dev, lo, hi)
            nbytes = int(w.k[lo:hi].astype(np.int64).sum()) * m.bytes_per_token
            timed("pack", lambda: kvm.kvm_pack(src_pool, sg, staging, staging_bytes=nbytes))
            timed("unpack", lambda: kvm.kvm_unpack(staging, dst_pool, dg, staging_bytes=nbytes))
        timed("migrate", lambda: kvm.kvm_migrate(src_pool, src_batch, dst_pool, dst_batch))
        done = torch.cuda.Event()
        done.record(stream)
        timed("decode", lambda: kvm.kvm_paged_decode(dst_pool, dst_batch, q_dev, out, workspace=ws,
                                                     workspace_bytes=ws_bytes))
        if events is not None:
            events.append(marks)
        # the source blocks may be released only once the copies have finished
        done.synchronize()
        src_fl.free(s_blk)
        # bookkeeping so that the next step starts from the same state
        src_fl.reserve(s_blk)
        dst_fl.free(ids)
        return ids

    for _ in range(a.warmup):
        step(None)
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(a.steps):
        ids = step(events)
    torch.cuda.synchronize()
    t_total = time.perf_counter() - t0
    ms_step = t_total * 1e3 / a.steps
    kern_ms = {n: float(np.mean([sum(e0.elapsed_time(e1) for nm, e0, e1 in marks if nm == n)
                                 for marks in events])) for n in names}
    log("step %.3f ms; kernels (ms): %s" % (ms_step, {k: round(v, 4) for k, v in kern_ms.items()}))

    # practical ceiling: a plain contiguous device-to-device copy of the same payload
    # (one half of the staging buffer copied onto the other: no extra allocation)
    nb16 = min(payload, stage_bytes // 2) // 16 * 16
    half_a, half_b = staging[:nb16], staging[nb16:2 * nb16]
    for _ in range(2):
        wl_device.plain_copy(half_b, half_a, nb16)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(5):
        wl_device.plain_copy(half_b, half_a, nb16)
    e1.record(stream)
    torch.cuda.synchronize()
    memcpy_gbs = 2 * nb16 * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9

    # end-state check on sampled blocks: destination equals source, source equals generator
    verified = None
    if not a.no_verify:
        run = m.H * m.B * m.D
        sp = src_mem.view(torch.int16).view(2 * m.L, w.n_blocks_src, run)
        dp = dst_mem.view(torch.int16).view(2 * m.L, w.n_blocks_dst, run)
        rng = np.random.default_rng(1)
        bad = 0
        for _ in range(16):
            r = int(rng.integers(len(w.k)))
            if nbk[r] == 0:
                continue
            j = int(rng.integers(nbk[r]))
            p = int(rng.integers(2 * m.L))
            ns = min(m.B, int(w.k[r]) - j * m.B)
            sblk = int(s_blk[s_off[r] + j])
            dblk = int(ids[d_off[r] + j])
            s_h = sp[p, sblk].cpu().numpy().view(np.uint16).reshape(m.H, m.B, m.D)
            d_h = dp[p, dblk].cpu().numpy().view(np.uint16).reshape(m.H, m.B, m.D)
            gen_s = wl.gen_block(w.seed, wl.STREAM_SRC, m, p, sblk)
            gen_d = wl.gen_block(w.seed, wl.STREAM_DST, m, p, dblk)
            ok = (np.array_equal(s_h, gen_s) and np.array_equal(d_h[:, :ns], gen_s[:, :ns])
                  and np.array_equal(d_h[:, ns:], gen_d[:, ns:]))
            bad += 0 if ok else 1
        verified = bad == 0
        log("sampled end-state check: %s" % ("ok" if verified else "%d MISMATCHES" % bad))

    # reference access patterns from arithmetic addresses (no tables): the ceilings the
    # memory system gives a kernel of the copy kernels' shape, over the same pools
    reference = None
    if not a.no_reference_legs:
        sink = torch.zeros(4, dtype=torch.int32, device=dev)
        legs = [  # name, mode, run bytes, source random, destination random, source / destination die rotation
            ("read_stream", wl_device.REF_READ, 4096, False, False, 0, 0),
            ("write_stream", wl_device.REF_WRITE, 4096, False, False, 0, 0),
            ("read_random_4k", wl_device.REF_READ, 4096, True, False, 0, 0),
            ("read_random_32k", wl_device.REF_READ, 32768, True, False, 0, 0),
            ("write_random_32k", wl_device.REF_WRITE, 32768, False, True, 0, 0),
            ("copy_stream", wl_device.REF_COPY, 32768, False, False, 0, 0),
            ("copy_random_src_32k", wl_device.REF_COPY, 32768, True, False, 0, 0),
            ("copy_random_dst_32k", wl_device.REF_COPY, 32768, False, True, 0, 0),
            ("copy_random_both_32k", wl_device.REF_COPY, 32768, True, True, 0, 0),
            # which 4 KiB pieces a die touches: workgroup c of a 32 KiB run takes chunk c
            # (every die one residue class of pieces), chunk c + 1 (another fixed class) or
            # chunk c + r in run r (a class that changes from run to run)
            ("read_stream_32k", wl_device.REF_READ, 32768, False, False, 0, 0),
            ("read_stream_32k_shifted", wl_device.REF_READ, 32768, False, False, 1, 0),
            ("read_stream_32k_varying", wl_device.REF_READ, 32768, False, False, 8, 0),
            ("write_stream_32k", wl_device.REF_WRITE, 32768, False, False, 0, 0),
            ("write_stream_32k_shifted", wl_device.REF_WRITE, 32768, False, False, 0, 1),
            ("write_stream_32k_varying", wl_device.REF_WRITE, 32768, False, False, 0, 8),
            ("copy_stream_src_varying", wl_device.REF_COPY, 32768, False, False, 8, 0),
            ("copy_stream_dst_varying", wl_device.REF_COPY, 32768, False, False, 0, 8),
            ("copy_stream_both_varying", wl_device.REF_COPY, 32768, False, False, 8, 8),
        ]
        reference = {}
        ref_bytes = min(payload, 8 << 30)      # enough for a steady rate; fits every pool's permuted slots

        def time_leg(name, fn, moved):
            for _ in range(2):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(5):
                fn()
            e1.record(stream)
            torch.cuda.synchronize()
            reference[name] = {"GB/s": round(moved * 5 / (e0.elapsed_time(e1) * 1e-3) / 1e9, 1),
                               "bytes": moved}

        for name, mode, run, rs, rd, srot, drot in legs:
            n_runs = ref_bytes // run
            args = (mode, src_mem if mode != wl_device.REF_WRITE else None,
                    dst_mem if mode != wl_device.REF_READ else None, run, n_runs, rs, rd, sink, srot, drot)
            time_leg(name, lambda: wl_device.ref_stream(*args),
                     n_runs * run * (2 if mode == wl_device.REF_COPY else 1))
        # the decode's read shape without its arithmetic: four waves walking sequences of
        # 4 KiB pieces, four K-like and four V-like pieces per step (sixteen steps, as a
        # context of 64 blocks), over the first 8 GiB of the source pool
        walk_mem = src_mem[:min(src_mem.numel(), 8 << 30)]
        walks = [  # name, pieces between the four pieces of a step, sliced
            ("walk_piece_per_wave_1m_apart", 256, False),
            ("walk_sliced_1m_apart", 256, True),
            ("walk_sliced_adjacent", 1, True),
            ("walk_sliced_32k_apart", 8, True),
            ("walk_sliced_128k_apart", 32, True),
            ("walk_sliced_512k_apart", 128, True),
            ("walk_sliced_4m_apart", 1024, True),
        ]
        for name, stride, sliced in walks:
            nbytes = wl_device.ref_walk(walk_mem, ref_bytes, stride, 16, sliced, sink)
            time_leg(name, lambda: wl_device.ref_walk(walk_mem, ref_bytes, stride, 16, sliced, sink), nbytes)
        log("reference legs (GB/s): %s" % {k: v["GB/s"] for k, v in reference.items()})

    value = 6 * payload / (ms_step * 1e-3) / 1e9
    mig_gbs = 2 * payload / (kern_ms["migrate"] * 1e-3) / 1e9
    result = {
        "metric": "KV migrate GB/s (read+write)",
        "value": round(value, 2),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": a.steps,
        "warmup": a.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u16",
        "data": "synthetic",
        "config": {
            "workload": w.name,
            "shape": "L%d H%d Hq%d D%d B%d %s" % (m.L, m.H, m.Hq, m.D, m.B, m.dtype),
            "pool_blocks": [w.n_blocks_src, w.n_blocks_dst],
            "live_requests": len(w.lens),
            "migrated_requests": len(w.k),
            "migrated_tokens": int(w.k.sum()),
            "migrated_blocks": n_dst,
            "payload_bytes": payload,
            "value_is": "bytes read+written by pack, unpack and fused migrate (6 x payload) per "
                        "second of whole-step time; the step also allocates, uploads the table, "
                        "runs paged decode over the destination (whose bytes are not counted) and "
                        "releases the source.  The >= 70 % of HBM peak target is quoted on the "
                        "fused migrate kernel alone: read it from roofline.frac",
            "notes": w.notes,
        },
        "frac_of_hbm_peak": round(value / HBM_PEAK_GBS, 4),
        "migrated_blocks_per_s": round(n_dst / (kern_ms["migrate"] * 1e-3), 1),
        "kernels": {
            "pack": {"ms": round(kern_ms["pack"], 4),
                     "GB/s": round(2 * payload / kern_ms["pack"] / 1e6, 1),
                     "frac_of_hbm_peak": round(2 * payload / kern_ms["pack"] / 1e6 / HBM_PEAK_GBS, 4)},
            "unpack": {"ms": round(kern_ms["unpack"], 4),
                       "GB/s": round(2 * payload / kern_ms["unpack"] / 1e6, 1),
                       "frac_of_hbm_peak": round(2 * payload / kern_ms["unpack"] / 1e6 / HBM_PEAK_GBS, 4)},
            "migrate": {"ms": round(kern_ms["migrate"], 4), "GB/s": round(mig_gbs, 1),
                        "frac_of_hbm_peak": round(mig_gbs / HBM_PEAK_GBS, 4)},
            "decode": {"ms": round(kern_ms["decode"], 4),
                       "GB/s": round(payload / kern_ms["decode"] / 1e6, 1),
                       "frac_of_hbm_peak": round(payload / kern_ms["decode"] / 1e6 / HBM_PEAK_GBS, 4)},
            "plain_copy": {"GB/s": round(memcpy_gbs, 1), "bytes": nb16},
        },
        "reference": reference,
        "verified": verified,
        "roofline": {
            "kernel": "copy_kernel<migrate> (kvm_migrate)",
            "bound": "hbm",
            "achieved": round(mig_gbs, 1),
            "peak": HBM_PEAK_GBS,
            "unit": "GB/s",
            "frac": round(mig_gbs / HBM_PEAK_GBS, 4),
            "traffic": measured_traffic(w.name, payload),
            "algorithmic_bytes": 2 * payload,
        },
    }
    if not a.no_cpu_baseline:
        del staging
        result["cpu_baseline"] = cpu_baseline(w, src_mem, m.bytes_per_token, a.cpu_sample, log)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
