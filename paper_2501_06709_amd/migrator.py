"""Host-side sequencing of migration orders around the library calls.

An order moves tokens [0,k) of one request from its pool into another pool of the
same model (arXiv 2501.06709, Sec. "Adaptive Request Migration"): pop the
destination blocks from the destination free list, get both block tables to the
device, enqueue kvm_migrate (and optionally paged decode over the destination),
and return the source blocks to the source free list only after the copy has
finished ("Boundary Profiling": source memory is held until the transfer is
complete).

Orders are staged first and enqueued together (`stage` ... `flush`).  The
scheduler hands over a time slot's move list at once (Sec. "Online KV Cache
Scheduling", request operation batching), so the orders of a slot are known
together, and a flush turns them into few, large launches:
  * the tables of all staged orders travel in ONE host-to-device copy;
  * the staged orders that share a (source pool, destination pool) pair become ONE
    kvm_migrate call and ONE kvm_paged_decode_rows call (the kernels carry 64
    requests per launch) - single-request launches of a few thousand workgroups
    spend much of their time filling and draining the chip;
  * one event per flush; the source blocks of its orders are released once that
    event has completed (at most `depth` flushes are in flight before the host
    waits for the oldest), so the stream never drains between flushes.
An order whose source blocks are written by an order that is still staged (the same
request moved twice) cannot share a launch with it: staging it flushes first.

All data movement happens in the library's kernels; this module only orders the
calls and keeps the integer bookkeeping.
"""
from collections import deque

import numpy as np
import torch

from . import binding as kvm


class DevicePool:
    """A block pool on the device with its free list."""

    def __init__(self, mem_or_addr, n_blocks, layout, occupied=None):
        self.pool = kvm.Pool(mem_or_addr, n_blocks, layout)
        self.layout = layout
        self.n_blocks = n_blocks
        self.free = kvm.FreeList(n_blocks, occupied)
        # blocks that a staged, not yet enqueued order will write
        self.staged_writes = np.zeros(n_blocks, dtype=bool)


class _Staged:
    __slots__ = ("table", "ids", "k", "src", "dst", "decode")

    def __init__(self, table, ids, k, src, dst, decode):
        self.table, self.ids, self.k, self.src, self.dst, self.decode = table, ids, k, src, dst, decode


class Migrator:
    """depth: flushes that may be in flight before the host waits for the oldest one
    (the source blocks of its orders are released then); max_staged: orders per flush
    (a full stage flushes by itself); decode_workspace: optional device buffer for
    splitting long decode contexts (shared by all decode calls, which run one after
    the other on the stream)."""

    def __init__(self, device, max_blocks_per_request, depth=4, max_staged=16, decode_workspace=None,
                 time_copies=False):
        self.device = device
        self.max_blocks = max_blocks_per_request
        self.depth = depth
        self.max_staged = max_staged
        self.ws = decode_workspace
        # table space: a ring of regions, one per flush; a region is rewritten only
        # after the flush that read it has finished
        self.region_ints = 2 * max_blocks_per_request * max_staged
        self.n_regions = depth + 2
        self.pin = torch.empty(self.n_regions * self.region_ints, dtype=torch.int32, pin_memory=True)
        self.dev = torch.empty(self.n_regions * self.region_ints, dtype=torch.int32, device=device)
        self.region_event = [None] * self.n_regions
        self.region = 0
        self.staged = []
        self.pending = deque()      # (event, [(source DevicePool, source ids)]) awaiting release
        self.launches = 0           # kvm_migrate + decode calls made so far
        # time_copies: an event pair around every kvm_migrate call -> (events, bytes read + written)
        self.copy_marks = [] if time_copies else None

    # ---- deferred source release ----
    def _retire_oldest(self):
        ev, released = self.pending.popleft()
        ev.synchronize()
        for src, ids in released:
            src.free.free(ids)

    def drain(self, stream=None):
        """Enqueue what is staged, wait for every order and release its source blocks."""
        self.flush(stream)
        while self.pending:
            self._retire_oldest()

    # ---- staging ----
    def stage(self, table, length, src, dst, k, decode=None):
        """Allocate the destination blocks of one order and note it for the next flush.

        Returns the new table (ids in `dst`).  Raises KvmError(KVM_ENOMEM) when `dst`
        cannot supply the blocks even after every finished order has released its
        source; nothing has been changed then.
        decode = (q_dev, out_dev, row): paged decode of this request over the
        destination right after its copy, query and output in row `row` of the two
        buffers ([rows][layers][query heads][head_dim]); orders staged together that
        decode from the same buffers need distinct rows.
        """
        B = src.layout.block_tokens
        nb = -(-int(k) // B)
        table = np.asarray(table, np.int32).copy()
        assert 0 <= k <= length and len(table) <= self.max_blocks
        if len(self.staged) >= self.max_staged or (len(table) and src.staged_writes[table].any()):
            self.flush()
        while len(self.pending) >= self.depth:
            self._retire_oldest()
        try:
            ids = dst.free.alloc(nb)                  # KVM_ENOMEM leaves everything as it was
        except kvm.KvmError as e:
            if e.status != kvm.KVM_ENOMEM:
                raise
            # blocks may be waiting for the release of orders that are still staged or in flight
            self.drain()
            ids = dst.free.alloc(nb)
        dst.staged_writes[ids] = True
        self.staged.append(_Staged(table, ids, int(k), src, dst, decode))
        return ids

    def flush(self, stream=None):
        """One upload for all staged orders, then one kvm_migrate and one decode call
        per (source pool, destination pool) pair, pairs in order of first appearance."""
        if not self.staged:
            return
        st = torch.cuda.current_stream() if stream is None else stream
        staged, self.staged = self.staged, []
        for o in staged:
            o.dst.staged_writes[o.ids] = False
        groups = {}
        for o in staged:
            groups.setdefault((id(o.src), id(o.dst)), []).append(o)
        # the region's previous readers must be done before it is rewritten
        ev = self.region_event[self.region]
        if ev is not None:
            ev.synchronize()
            self.region_event[self.region] = None
        lo = self.region * self.region_ints
        pin = self.pin.numpy()
        at = lo
        plans = []
        for members in groups.values():
            s_off = np.zeros(len(members) + 1, np.int32)
            d_off = np.zeros(len(members) + 1, np.int32)
            s_off[1:] = np.cumsum([len(o.table) for o in members])
            d_off[1:] = np.cumsum([len(o.ids) for o in members])
            s_blk = np.concatenate([o.table for o in members]) if s_off[-1] else np.zeros(0, np.int32)
            d_blk = np.concatenate([o.ids for o in members]) if d_off[-1] else np.zeros(0, np.int32)
            s_at, d_at = at, at + int(s_off[-1])
            pin[s_at:d_at] = s_blk
            pin[d_at:d_at + int(d_off[-1])] = d_blk
            at = d_at + int(d_off[-1])
            plans.append((members, s_off, s_blk, s_at, d_off, d_blk, d_at))
        # in-stream: an upload on a side stream with an event wait measured 15 us per
        # order slower than the copy it hides
        if at > lo:
            with torch.cuda.stream(st):
                self.dev[lo:at].copy_(self.pin[lo:at], non_blocking=True)
        released, failed = [], None
        for gi, (members, s_off, s_blk, s_at, d_off, d_blk, d_at) in enumerate(plans):
            ks = np.array([o.k for o in members], dtype=np.int32)
            src, dst = members[0].src, members[0].dst
            sb = kvm.Batch(s_off, s_blk, ks, self.dev[s_at:s_at + max(len(s_blk), 1)])
            db = kvm.Batch(d_off, d_blk, ks, self.dev[d_at:d_at + max(len(d_blk), 1)])
            try:
                if self.copy_marks is not None:
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(st)
                kvm.kvm_migrate(src.pool, sb, dst.pool, db, stream=st)
                if self.copy_marks is not None:
                    e1.record(st)
                    self.copy_marks.append((e0, e1, 2 * int(ks.sum()) * kvm.kvm_bytes_per_token(src.layout)))
                self.launches += 1
            except kvm.KvmError as e:
                # nothing of this group or of the later ones was enqueued: their
                # destination blocks go back at once, their sources stay allocated
                for later in plans[gi:]:
                    for o in later[0]:
                        o.dst.free.free(o.ids)
                failed = e
                break
            # from here on the group's copy is in flight: its sources are released
            # after the flush's event, whatever happens to the decode call
            released += [(o.src, o.table) for o in members]
            try:
                self._decode_group(members, dst, db, st)
            except kvm.KvmError as e:
                for later in plans[gi + 1:]:
                    for o in later[0]:
                        o.dst.free.free(o.ids)
                failed = e
                break
        ev = torch.cuda.Event()
        ev.record(st)
        if released:
            self.pending.append((ev, released))
        self.region_event[self.region] = ev
        self.region = (self.region + 1) % self.n_regions
        if failed is not None:
            raise failed

    def _decode_group(self, members, dst, db, st):
        """Decode of the group's requests over the destination: one call per distinct
        (q, out) buffer pair, normally one."""
        by_buf = {}
        for i, o in enumerate(members):
            if o.decode is not None and o.k > 0:
                q_dev, out_dev, row = o.decode
                by_buf.setdefault((q_dev.data_ptr(), out_dev.data_ptr()), (q_dev, out_dev, []))[2].append((i, row))
        for q_dev, out_dev, picks in by_buf.values():
            rows = np.zeros(len(members), np.int32)
            ks = np.zeros(len(members), np.int32)       # requests without a decode: k = 0, skipped
            for i, row in picks:
                rows[i], ks[i] = row, members[i].k
            batch = kvm.Batch(db.offsets, db.blocks, ks, db.blocks_dev)
            kvm.kvm_paged_decode_rows(dst.pool, batch, rows, q_dev, out_dev, workspace=self.ws, stream=st)
            self.launches += 1

    def move(self, table, length, src, dst, k, decode=None, stream=None):
        """Stage and enqueue one order at once; returns the new table."""
        ids = self.stage(table, length, src, dst, k, decode)
        self.flush(stream)
        return ids
