"""Python face of the library's order sequencer (kvm_sequencer_* in kvm.h).

An order moves tokens [0,k) of one request from its pool into another pool of the
same model (arXiv 2501.06709, Sec. "Adaptive Request Migration").  The sequencing
itself - destination allocation, one table upload per flush, one kvm_migrate and
one kvm_paged_decode_rows call per (source pool, destination pool) pair of a
flush, release of the source blocks only after the flush's event has completed -
lives in the library; this module marshals arguments and owns the buffers the
sequencer needs (a pinned host buffer and a device buffer for the block tables).
"""
import ctypes

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


class Migrator:
    """depth: flushes that may be in flight before a call waits for the oldest one
    (the source blocks of its orders are released then); max_staged: orders per flush
    (a full stage flushes by itself); decode_workspace: optional device buffer for
    splitting long decode contexts; time_copies: bracket every kvm_migrate call with
    HIP events (see copy_stats)."""

    def __init__(self, device, max_blocks_per_request, depth=4, max_staged=16, decode_workspace=None,
                 time_copies=False):
        L = kvm.lib()
        self.device = device
        self.max_blocks = int(max_blocks_per_request)
        n = L.kvm_sequencer_table_ints(self.max_blocks, int(max_staged), int(depth))
        if n < 0:
            raise kvm.KvmError(kvm.KVM_EINVAL, "bad sequencer sizes")
        self.pin = torch.empty(n, dtype=torch.int32, pin_memory=True)
        self.dev = torch.empty(n, dtype=torch.int32, device=device)
        self.ws = decode_workspace
        ws_bytes = decode_workspace.numel() * decode_workspace.element_size() if decode_workspace is not None else 0
        self._h = L.kvm_sequencer_create(self.max_blocks, int(max_staged), int(depth), self.pin.data_ptr(),
                                         self.dev.data_ptr(), n, kvm._devptr(decode_workspace), ws_bytes)
        if not self._h:
            raise kvm.KvmError(kvm.KVM_EINVAL, L.kvm_last_error().decode())
        if time_copies:
            kvm._check(L.kvm_sequencer_timing(self._h, 1))
        self._keep = []       # q / out tensors of staged orders, kept alive until the next drain
        self._pools = {}      # pools (and their free lists) the sequencer may still refer to

    @property
    def launches(self):
        """kvm_migrate + decode calls made so far."""
        return kvm.lib().kvm_sequencer_launches(self._h)

    def stage(self, table, length, src, dst, k, decode=None, stream=None):
        """Allocate the destination blocks of one order and note it for the next flush.

        Returns the new table (ids in `dst`).  Raises KvmError(KVM_ENOMEM) when `dst`
        cannot supply the blocks even after everything in flight has been released;
        nothing has been changed then.
        decode = (q_dev, out_dev, row): paged decode of this request over the
        destination right after its copy, query and float32 output in row `row` of the
        two buffers ([rows][layers][query heads][head_dim]); orders staged together
        that decode from the same buffers need distinct rows.
        """
        table = np.ascontiguousarray(table, dtype=np.int32)
        assert 0 <= k <= length
        nb = -(-int(k) // src.layout.block_tokens)
        out = np.empty(nb, dtype=np.int32)
        q_dev, out_dev, row = decode if decode is not None else (None, None, 0)
        kvm._check(kvm.lib().kvm_sequencer_stage(
            self._h, ctypes.byref(src.pool.c), src.free._h, ctypes.byref(dst.pool.c), dst.free._h,
            table.ctypes.data, len(table), int(k), kvm._devptr(q_dev), kvm._devptr(out_dev), int(row),
            out.ctypes.data, kvm._stream(stream)))
        self._pools[id(src)] = src
        self._pools[id(dst)] = dst
        if decode is not None:
            self._keep.append((q_dev, out_dev))
        return out

    def flush(self, stream=None):
        """Enqueue everything staged: one upload, then one kvm_migrate and one decode
        call per (source pool, destination pool) pair."""
        kvm._check(kvm.lib().kvm_sequencer_flush(self._h, kvm._stream(stream)))

    def drain(self, stream=None):
        """Enqueue what is staged, wait for every order and release its source blocks."""
        kvm._check(kvm.lib().kvm_sequencer_drain(self._h, kvm._stream(stream)))
        self._keep.clear()

    def move(self, table, length, src, dst, k, decode=None, stream=None):
        """Stage and enqueue one order at once; returns the new table."""
        ids = self.stage(table, length, src, dst, k, decode, stream)
        self.flush(stream)
        return ids

    def copy_stats(self):
        """(milliseconds, bytes read + written, launches) of the timed kvm_migrate calls."""
        ms, nbytes, n = ctypes.c_double(), ctypes.c_int64(), ctypes.c_int64()
        kvm._check(kvm.lib().kvm_sequencer_copy_stats(self._h, ctypes.byref(ms), ctypes.byref(nbytes),
                                                      ctypes.byref(n)))
        return ms.value, nbytes.value, n.value

    def reset_copy_stats(self):
        kvm._check(kvm.lib().kvm_sequencer_timing(self._h, 1))

    def close(self):
        if self._h:
            kvm.lib().kvm_sequencer_destroy(self._h)   # waits, releases sources into the free lists
            self._h = None
        self._pools.clear()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
