"""Host-side sequencing of migration orders around the library calls.

An order moves tokens [0,k) of one request from its pool into another pool of the
same model (arXiv 2501.06709, Sec. "Adaptive Request Migration"): pop the
destination blocks from the destination free list, get both block tables to the
device, enqueue kvm_migrate (and optionally kvm_paged_decode over the
destination), and return the source blocks to the source free list only after the
copy has finished ("Boundary Profiling": source memory is held until the transfer
is complete).  Orders are enqueued back to back on one stream; the release of an
order is deferred until its event has completed, so the stream never drains
between orders.

Orders can be staged first and enqueued together (`stage` ... `flush`): the
tables of all staged orders then travel in ONE host-to-device copy.  On the GPU a
table copy between two orders costs about 11 us (a small copy kernel and the
dependencies around it), a tenth of a typical order of the mixed workload; the
scheduler hands over a time slot's move list at once (Sec. "Online KV Cache
Scheduling", request operation batching), so the lists are known together.

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


class _Staged:
    __slots__ = ("table", "ids", "k", "src", "dst", "decode", "at")

    def __init__(self, table, ids, k, src, dst, decode, at):
        self.table, self.ids, self.k, self.src, self.dst, self.decode, self.at = table, ids, k, src, dst, decode, at


class Migrator:
    """depth: orders that may be in flight before the host waits for the oldest one
    (its source blocks are released then); max_staged: orders per table upload."""

    def __init__(self, device, max_blocks_per_request, depth=4, max_staged=16):
        self.device = device
        self.max_blocks = max_blocks_per_request
        self.depth = depth
        self.max_staged = max_staged
        # table space: a ring of regions, one per flush; a region is rewritten only
        # after the last order that read it has finished
        self.region_ints = 2 * max_blocks_per_request * max_staged
        self.n_regions = depth + 2
        self.pin = torch.empty(self.n_regions * self.region_ints, dtype=torch.int32, pin_memory=True)
        self.dev = torch.empty(self.n_regions * self.region_ints, dtype=torch.int32, device=device)
        self.region_event = [None] * self.n_regions
        self.region = 0
        self.fill = 0               # ints used in the current region
        self.staged = []
        self.pending = deque()      # (event, source DevicePool, source ids) awaiting release

    # ---- deferred source release ----
    def _retire_oldest(self):
        ev, src, ids = self.pending.popleft()
        ev.synchronize()
        src.free.free(ids)

    def drain(self):
        """Enqueue what is staged, wait for every order and release its source blocks."""
        self.flush()
        while self.pending:
            self._retire_oldest()

    # ---- staging ----
    def stage(self, table, length, src, dst, k, decode=None):
        """Allocate the destination blocks of one order and note it for the next flush.

        Returns the new table (ids in `dst`).  Raises KvmError(KVM_ENOMEM) when `dst`
        cannot supply the blocks; nothing has been changed then.
        decode = (q_dev, out_dev, ws_dev, ws_bytes) runs paged decode of this request
        over the destination right after its copy.
        """
        B = src.layout.block_tokens
        nb = -(-int(k) // B)
        n_src = len(table)
        assert 0 <= k <= length and n_src <= self.max_blocks
        if len(self.staged) >= self.max_staged:
            self.flush()
        while len(self.pending) >= self.depth:
            self._retire_oldest()
        if not self.staged:
            # first order of a region: the region's previous readers must be done
            ev = self.region_event[self.region]
            if ev is not None:
                ev.synchronize()
                self.region_event[self.region] = None
        ids = dst.free.alloc(nb)                      # KVM_ENOMEM leaves everything as it was
        table = np.asarray(table, np.int32).copy()
        at = self.region * self.region_ints + self.fill
        pin = self.pin.numpy()
        pin[at:at + n_src] = table
        pin[at + n_src:at + n_src + nb] = ids
        self.fill += n_src + nb
        self.staged.append(_Staged(table, ids, int(k), src, dst, decode, at))
        return ids

    def flush(self, stream=None):
        """One upload for all staged orders, then their kernels in staging order."""
        if not self.staged:
            return
        st = torch.cuda.current_stream() if stream is None else stream
        lo = self.region * self.region_ints
        # in-stream: an upload on a side stream with an event wait measured 15 us per
        # order slower than the copy it hides
        with torch.cuda.stream(st):
            self.dev[lo:lo + self.fill].copy_(self.pin[lo:lo + self.fill], non_blocking=True)
        staged, self.staged = self.staged, []
        ev = None
        try:
            for i, o in enumerate(staged):
                n_src, nb = len(o.table), len(o.ids)
                src_dev = self.dev[o.at:o.at + max(n_src, 1)]
                dst_dev = self.dev[o.at + n_src:o.at + n_src + max(nb, 1)]
                ks = np.array([o.k], dtype=np.int32)
                sb = kvm.Batch(np.array([0, n_src], np.int32), o.table, ks, src_dev)
                db = kvm.Batch(np.array([0, nb], np.int32), o.ids, ks, dst_dev)
                kvm.kvm_migrate(o.src.pool, sb, o.dst.pool, db, stream=st)
                if o.decode is not None and o.k > 0:
                    q_dev, out_dev, ws_dev, ws_bytes = o.decode
                    kvm.kvm_paged_decode(o.dst.pool, db, q_dev, out_dev, workspace=ws_dev,
                                         workspace_bytes=ws_bytes, stream=st)
                ev = torch.cuda.Event()
                ev.record(st)
                self.pending.append((ev, o.src, o.table))
        except kvm.KvmError:
            # orders that were not enqueued give their destination blocks back
            for o in staged[i:]:
                o.dst.free.free(o.ids)
            raise
        finally:
            if ev is None:
                ev = torch.cuda.Event()
                ev.record(st)
            self.region_event[self.region] = ev
            self.region = (self.region + 1) % self.n_regions
            self.fill = 0

    def move(self, table, length, src, dst, k, decode=None, stream=None):
        """Stage and enqueue one order at once; returns the new table."""
        ids = self.stage(table, length, src, dst, k, decode)
        self.flush(stream)
        return ids
