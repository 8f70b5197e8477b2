"""ctypes binding of libkvm.so: argument marshalling only.

Every step of the migration path runs in the library's HIP kernels; this module
turns numpy arrays and torch tensors (used purely as owners of device memory)
into the plain structs and pointers of ``include/kvm.h`` and raises
:class:`KvmError` on a negative status.  There is no fallback: if the library
has not been built, loading raises.
"""
import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvm.so")

KVM_OK, KVM_EINVAL, KVM_ENOMEM, KVM_EHIP = 0, -1, -2, -3
KVM_F16, KVM_BF16 = 0, 1
DTYPES = {"f16": KVM_F16, "bf16": KVM_BF16}


class KvmError(RuntimeError):
    def __init__(self, status, detail):
        super().__init__("kvm status %d: %s" % (status, detail))
        self.status = status
        self.detail = detail


class kvm_layout(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("n_q_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("block_tokens", ctypes.c_int32), ("dtype", ctypes.c_int32),
                ("stride_layer", ctypes.c_int64), ("stride_kv", ctypes.c_int64),
                ("stride_block", ctypes.c_int64), ("stride_head", ctypes.c_int64),
                ("stride_slot", ctypes.c_int64)]


class kvm_pool(ctypes.Structure):
    _fields_ = [("base", ctypes.c_void_p), ("n_blocks", ctypes.c_int64), ("layout", kvm_layout)]


class kvm_batch(ctypes.Structure):
    _fields_ = [("n_req", ctypes.c_int32), ("bt_offsets", ctypes.c_void_p),
                ("bt_blocks_dev", ctypes.c_void_p), ("bt_blocks_host", ctypes.c_void_p),
                ("k", ctypes.c_void_p), ("start", ctypes.c_void_p)]


_lib = None


def lib():
    """The loaded library; raises if it was not built (no silent fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libkvm.so is missing: run __graft_entry__.build() "
                               "(python -m paper_2501_06709_amd.build) first")
        L = ctypes.CDLL(LIB_PATH)
        P, I32, I64, VP = ctypes.POINTER, ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
        L.kvm_bytes_per_token.restype = I64
        L.kvm_bytes_per_token.argtypes = [P(kvm_layout)]
        L.kvm_block_bytes.restype = I64
        L.kvm_block_bytes.argtypes = [P(kvm_layout)]
        L.kvm_staging_bytes.restype = I64
        L.kvm_staging_bytes.argtypes = [P(kvm_layout), P(kvm_batch)]
        L.kvm_layout_canonical.restype = ctypes.c_int
        L.kvm_layout_canonical.argtypes = [P(kvm_layout), I32, I32, I32, I32, I32, I32, I64]
        L.kvm_pool_span_bytes.restype = I64
        L.kvm_pool_span_bytes.argtypes = [P(kvm_layout), I64]
        L.kvm_pack.restype = ctypes.c_int
        L.kvm_pack.argtypes = [P(kvm_pool), P(kvm_batch), VP, I64, VP]
        L.kvm_unpack.restype = ctypes.c_int
        L.kvm_unpack.argtypes = [VP, I64, P(kvm_pool), P(kvm_batch), VP]
        L.kvm_migrate.restype = ctypes.c_int
        L.kvm_migrate.argtypes = [P(kvm_pool), P(kvm_batch), P(kvm_pool), P(kvm_batch), VP]
        L.kvm_paged_decode.restype = ctypes.c_int
        L.kvm_paged_decode.argtypes = [P(kvm_pool), P(kvm_batch), VP, VP, ctypes.c_int,
                                       ctypes.c_float, VP, I64, VP]
        L.kvm_paged_decode_rows.restype = ctypes.c_int
        L.kvm_paged_decode_rows.argtypes = [P(kvm_pool), P(kvm_batch), VP, VP, VP, ctypes.c_int,
                                            ctypes.c_float, VP, I64, VP]
        L.kvm_paged_decode_static.restype = ctypes.c_int
        L.kvm_paged_decode_static.argtypes = [P(kvm_pool), P(kvm_batch), VP, VP, ctypes.c_int,
                                              ctypes.c_float, VP]
        L.kvm_decode_workspace_bytes.restype = I64
        L.kvm_decode_workspace_bytes.argtypes = [P(kvm_layout), P(kvm_batch)]
        L.kvm_freelist_create.restype = VP
        L.kvm_freelist_create.argtypes = [I64, VP]
        L.kvm_freelist_destroy.restype = None
        L.kvm_freelist_destroy.argtypes = [VP]
        L.kvm_freelist_available.restype = I64
        L.kvm_freelist_available.argtypes = [VP]
        L.kvm_freelist_alloc.restype = ctypes.c_int
        L.kvm_freelist_alloc.argtypes = [VP, I32, VP]
        L.kvm_freelist_free.restype = ctypes.c_int
        L.kvm_freelist_free.argtypes = [VP, I32, VP]
        L.kvm_freelist_reserve.restype = ctypes.c_int
        L.kvm_freelist_reserve.argtypes = [VP, I32, VP]
        L.kvm_divide_moves.restype = ctypes.c_int
        L.kvm_divide_moves.argtypes = [VP, I32, VP, I32, VP, I32, I32, VP]
        L.kvm_sequencer_table_ints.restype = I64
        L.kvm_sequencer_table_ints.argtypes = [I32, I32, I32]
        L.kvm_sequencer_create.restype = VP
        L.kvm_sequencer_create.argtypes = [I32, I32, I32, VP, VP, I64, VP, I64]
        L.kvm_sequencer_destroy.restype = None
        L.kvm_sequencer_destroy.argtypes = [VP]
        L.kvm_sequencer_stage.restype = ctypes.c_int
        L.kvm_sequencer_stage.argtypes = [VP, P(kvm_pool), VP, P(kvm_pool), VP, VP, I32, I32, VP, VP, I32, VP, VP]
        L.kvm_sequencer_flush.restype = ctypes.c_int
        L.kvm_sequencer_flush.argtypes = [VP, VP]
        L.kvm_sequencer_drain.restype = ctypes.c_int
        L.kvm_sequencer_drain.argtypes = [VP, VP]
        L.kvm_sequencer_launches.restype = I64
        L.kvm_sequencer_launches.argtypes = [VP]
        L.kvm_sequencer_timing.restype = ctypes.c_int
        L.kvm_sequencer_timing.argtypes = [VP, ctypes.c_int]
        L.kvm_sequencer_copy_stats.restype = ctypes.c_int
        L.kvm_sequencer_copy_stats.argtypes = [VP, P(ctypes.c_double), P(I64), P(I64)]
        L.kvm_strerror.restype = ctypes.c_char_p
        L.kvm_strerror.argtypes = [ctypes.c_int]
        L.kvm_last_error.restype = ctypes.c_char_p
        L.kvm_last_error.argtypes = []
        L.kvm_set_option.restype = ctypes.c_int
        L.kvm_set_option.argtypes = [ctypes.c_char_p, I64]
        _lib = L
    return _lib


def _check(status):
    if status < 0:
        L = lib()
        detail = L.kvm_last_error().decode() or L.kvm_strerror(status).decode()
        raise KvmError(status, detail)
    return status


def _devptr(x):
    """Device address of a torch tensor (or a plain int / None)."""
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return x.data_ptr()


def _stream(stream):
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def kvm_layout_canonical(n_layers, n_kv_heads, n_q_heads, head_dim, block_tokens, dtype, n_blocks):
    out = kvm_layout()
    _check(lib().kvm_layout_canonical(ctypes.byref(out), n_layers, n_kv_heads, n_q_heads, head_dim,
                                      block_tokens, DTYPES.get(dtype, dtype), n_blocks))
    return out


def kvm_bytes_per_token(layout):
    return lib().kvm_bytes_per_token(ctypes.byref(layout))


def kvm_block_bytes(layout):
    return lib().kvm_block_bytes(ctypes.byref(layout))


def kvm_pool_span_bytes(layout, n_blocks):
    return lib().kvm_pool_span_bytes(ctypes.byref(layout), n_blocks)


class Pool:
    """A block pool: a device buffer (torch tensor or address) plus its layout."""

    def __init__(self, mem, n_blocks, layout):
        self.mem = mem  # keeps the tensor alive
        self.n_blocks = int(n_blocks)
        self.layout = layout
        self.c = kvm_pool(_devptr(mem), self.n_blocks, layout)


class Batch:
    """CSR block tables of a batch.  `blocks_dev` is a device int32 buffer with
    the same ids as `blocks` (host); `host_ids=False` withholds the host copy so
    the library skips its id checks; `start` (optional) makes every call move only
    tokens [start[r], k[r])."""

    def __init__(self, offsets, blocks, k, blocks_dev, host_ids=True, start=None):
        self.offsets = np.ascontiguousarray(offsets, dtype=np.int32)
        self.blocks = np.ascontiguousarray(blocks, dtype=np.int32)
        self.k = np.ascontiguousarray(k, dtype=np.int32)
        self.start = None if start is None else np.ascontiguousarray(start, dtype=np.int32)
        assert self.start is None or len(self.start) == len(self.k)
        self.blocks_dev = blocks_dev
        self.n_req = len(self.k)
        assert len(self.offsets) == self.n_req + 1
        self.c = kvm_batch(self.n_req, self.offsets.ctypes.data, _devptr(blocks_dev),
                           self.blocks.ctypes.data if host_ids else None, self.k.ctypes.data,
                           None if self.start is None else self.start.ctypes.data)


def kvm_staging_bytes(layout, batch):
    return lib().kvm_staging_bytes(ctypes.byref(layout), ctypes.byref(batch.c))


def kvm_pack(src, src_reqs, staging, staging_bytes=None, stream=None):
    if staging_bytes is None:
        staging_bytes = staging.numel() * staging.element_size()
    return _check(lib().kvm_pack(ctypes.byref(src.c), ctypes.byref(src_reqs.c), _devptr(staging),
                                 staging_bytes, _stream(stream)))


def kvm_unpack(staging, dst, dst_reqs, staging_bytes=None, stream=None):
    if staging_bytes is None:
        staging_bytes = staging.numel() * staging.element_size()
    return _check(lib().kvm_unpack(_devptr(staging), staging_bytes, ctypes.byref(dst.c),
                                   ctypes.byref(dst_reqs.c), _stream(stream)))


def kvm_migrate(src, src_reqs, dst, dst_reqs, stream=None):
    return _check(lib().kvm_migrate(ctypes.byref(src.c), ctypes.byref(src_reqs.c),
                                    ctypes.byref(dst.c), ctypes.byref(dst_reqs.c), _stream(stream)))


def kvm_decode_workspace_bytes(layout, reqs):
    return lib().kvm_decode_workspace_bytes(ctypes.byref(layout), ctypes.byref(reqs.c))


def kvm_paged_decode(pool, reqs, q, out, out_is_f32=True, scale=0.0, workspace=None,
                     workspace_bytes=None, stream=None):
    if workspace is not None and workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    return _check(lib().kvm_paged_decode(ctypes.byref(pool.c), ctypes.byref(reqs.c), _devptr(q),
                                         _devptr(out), 1 if out_is_f32 else 0, scale,
                                         _devptr(workspace), workspace_bytes or 0, _stream(stream)))


def kvm_paged_decode_rows(pool, reqs, rows, q, out, out_is_f32=True, scale=0.0, workspace=None,
                          workspace_bytes=None, stream=None):
    rows = np.ascontiguousarray(rows, dtype=np.int32)
    assert len(rows) == reqs.n_req
    if workspace is not None and workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    return _check(lib().kvm_paged_decode_rows(ctypes.byref(pool.c), ctypes.byref(reqs.c), rows.ctypes.data,
                                              _devptr(q), _devptr(out), 1 if out_is_f32 else 0, scale,
                                              _devptr(workspace), workspace_bytes or 0, _stream(stream)))


KVM_STATIC_SCRATCH_BYTES = 32 << 20  # as in kvm.h


def kvm_paged_decode_static(pool, reqs, q, out, out_is_f32=True, scale=0.0, stream=None):
    return _check(lib().kvm_paged_decode_static(ctypes.byref(pool.c), ctypes.byref(reqs.c), _devptr(q),
                                                _devptr(out), 1 if out_is_f32 else 0, scale,
                                                _stream(stream)))


KVM_CLASS_KV, KVM_CLASS_TOKENS, KVM_CLASS_DEFER = 0, 1, 2
KVM_FIRST_FIT, KVM_BEST_FIT = 0, 1
MOVE_DTYPE = np.dtype([("link", np.int32), ("dst", np.int32), ("kv_bytes", np.int64),
                       ("tokens", np.int64)])


def kvm_divide_moves(moves, comm_boundary, comp_boundary, policy=KVM_FIRST_FIT):
    """moves: sequence of (link, dst, kv_bytes, tokens); returns int32 classes."""
    mv = np.array([tuple(m) for m in moves], dtype=MOVE_DTYPE) if len(moves) else np.zeros(0, MOVE_DTYPE)
    comm = np.ascontiguousarray(comm_boundary, dtype=np.int64)
    comp = np.ascontiguousarray(comp_boundary, dtype=np.int64)
    out = np.full(len(mv), -1, dtype=np.int32)
    _check(lib().kvm_divide_moves(mv.ctypes.data if len(mv) else None, len(mv),
                                  comm.ctypes.data if len(comm) else None, len(comm),
                                  comp.ctypes.data if len(comp) else None, len(comp),
                                  int(policy), out.ctypes.data if len(mv) else None))
    return out


def kvm_set_option(name, value):
    return _check(lib().kvm_set_option(name.encode(), int(value)))


class FreeList:
    """Host free list of a pool (kvm_freelist_*): lowest id first, all-or-nothing."""

    def __init__(self, n_blocks, occupied=None):
        occ = None
        if occupied is not None:
            occ = np.ascontiguousarray(occupied, dtype=np.uint8)
            assert len(occ) == n_blocks
        self._h = lib().kvm_freelist_create(int(n_blocks), occ.ctypes.data if occ is not None else None)
        if not self._h:
            raise KvmError(KVM_EINVAL, "kvm_freelist_create failed")

    def available(self):
        return lib().kvm_freelist_available(self._h)

    def alloc(self, n):
        out = np.empty(n, dtype=np.int32)
        _check(lib().kvm_freelist_alloc(self._h, int(n), out.ctypes.data))
        return out

    def free(self, ids):
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        _check(lib().kvm_freelist_free(self._h, len(ids), ids.ctypes.data))

    def reserve(self, ids):
        ids = np.ascontiguousarray(ids, dtype=np.int32)
        _check(lib().kvm_freelist_reserve(self._h, len(ids), ids.ctypes.data))

    def close(self):
        if self._h:
            lib().kvm_freelist_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
