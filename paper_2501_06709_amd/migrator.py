"""Host-side sequencing of one migration order around the library calls.

An order moves tokens [0,k) of one request from its pool into another pool of the
same model (arXiv 2501.06709, Sec. "Adaptive Request Migration"): pop the
destination blocks from the destination free list, upload both block tables
(one copy), enqueue kvm_migrate (and optionally kvm_paged_decode over the destination), and
return the source blocks to the source free list only after the copy has
finished ("Boundary Profiling": source memory is held until the transfer is
complete).  Orders are enqueued back to back on one stream; the release of order
i is deferred until its event has completed, which is checked when a later order
needs the slot, so the stream never drains between orders.

All data movement happens in the library's kernels; this module only orders the
calls and keeps the integer bookkeeping.
"""
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


class _Slot:
    """Pinned and device table space for one order in flight: the source table at
    [0, n_src), the destination table right behind it, so one copy uploads both."""

    def __init__(self, max_blocks, device):
        self.pin = torch.empty(2 * max_blocks, dtype=torch.int32, pin_memory=True)
        self.dev = torch.empty(2 * max_blocks, dtype=torch.int32, device=device)
        self.event = torch.cuda.Event()      # the order's kernels have finished
        self.pending = None  # (source DevicePool, source ids) awaiting release


class Migrator:
    def __init__(self, device, max_blocks_per_request, depth=4):
        self.device = device
        self.max_blocks = max_blocks_per_request
        self.slots = [_Slot(max_blocks_per_request, device) for _ in range(depth)]
        self.next = 0

    def _retire(self, slot):
        if slot.pending is not None:
            slot.event.synchronize()
            src, ids = slot.pending
            src.free.free(ids)
            slot.pending = None

    def drain(self):
        """Wait for every enqueued order and release its source blocks."""
        for s in self.slots:
            self._retire(s)

    def move(self, table, length, src, dst, k, decode=None, stream=None):
        """Enqueue the move of tokens [0,k) of a request whose blocks `table` (host
        int32 ids, covering `length` tokens) live in `src` into `dst`.

        Returns the new table (ids in `dst`).  Raises KvmError(KVM_ENOMEM) when
        `dst` cannot supply the blocks; nothing has been changed then.
        decode = (q_dev, out_dev, ws_dev, ws_bytes, row) runs paged decode of this
        request over the destination right after the copy.
        """
        B = src.layout.block_tokens
        nb = -(-int(k) // B)
        assert 0 <= k <= length and len(table) <= self.max_blocks
        slot = self.slots[self.next]
        self.next = (self.next + 1) % len(self.slots)
        self._retire(slot)
        ids = dst.free.alloc(nb)                      # KVM_ENOMEM leaves everything as it was
        st = torch.cuda.current_stream() if stream is None else stream
        n_src = len(table)
        pin = slot.pin.numpy()
        pin[:n_src] = table
        pin[n_src:n_src + nb] = ids
        n_up = max(n_src + nb, 1)
        # in-stream: an upload on a side stream with an event wait measured 15 us per
        # order slower than the copy it hides
        with torch.cuda.stream(st):
            slot.dev[:n_up].copy_(slot.pin[:n_up], non_blocking=True)
        src_dev, dst_dev = slot.dev[:max(n_src, 1)], slot.dev[n_src:n_src + max(nb, 1)]
        ks = np.array([k], dtype=np.int32)
        sb = kvm.Batch(np.array([0, n_src], np.int32), np.asarray(table, np.int32), ks, src_dev)
        db = kvm.Batch(np.array([0, nb], np.int32), ids, ks, dst_dev)
        try:
            kvm.kvm_migrate(src.pool, sb, dst.pool, db, stream=st)
            if decode is not None and k > 0:
                q_dev, out_dev, ws_dev, ws_bytes = decode
                kvm.kvm_paged_decode(dst.pool, db, q_dev, out_dev, workspace=ws_dev,
                                     workspace_bytes=ws_bytes, stream=st)
        except kvm.KvmError:
            dst.free.free(ids)
            raise
        slot.event.record(st)
        slot.pending = (src, np.asarray(table, np.int32).copy())
        return ids
