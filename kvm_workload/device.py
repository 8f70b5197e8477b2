"""Device-side helpers of the input generator (torch used for memory only)."""
import ctypes
import os
import subprocess

import numpy as np

from . import canonical_strides

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "fill.hip")
_LIB = os.path.join(_HERE, "libkvm_workload.so")
_lib = None


def build():
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    subprocess.check_call([hipcc, "--offload-arch=gfx950", "-O3", "-fPIC", "-shared",
                           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
                           _SRC, "-o", _LIB])
    return _LIB


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            raise RuntimeError("libkvm_workload.so is missing: run __graft_entry__.build() first")
        _lib = ctypes.CDLL(_LIB)
        _lib.kvmw_fill_pool.restype = ctypes.c_int
        _lib.kvmw_fill_pool.argtypes = [ctypes.c_void_p, ctypes.c_void_p] + [ctypes.c_int] * 5 + [
            ctypes.c_int64, ctypes.c_int64, ctypes.c_uint32, ctypes.c_uint32, ctypes.c_void_p]
        _lib.kvmw_gen_blocks.restype = ctypes.c_int
        _lib.kvmw_gen_blocks.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64] + [
            ctypes.c_int] * 4 + [ctypes.c_uint32] * 3 + [ctypes.c_void_p]
        _lib.kvmw_block_hashes.restype = ctypes.c_int
        _lib.kvmw_block_hashes.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int64,
                                           ctypes.c_int64, ctypes.c_void_p, ctypes.c_void_p]
        _lib.kvmw_ref_stream.restype = ctypes.c_int
        _lib.kvmw_ref_stream.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                                         ctypes.c_int64, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                         ctypes.c_void_p, ctypes.c_void_p]
        _lib.kvmw_ref_walk.restype = ctypes.c_int
        _lib.kvmw_ref_walk.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
                                       ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p]
        _lib.kvmw_plain_copy.restype = ctypes.c_int
        _lib.kvmw_plain_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64,
                                         ctypes.c_void_p]
    return _lib


def plain_copy(dst, src, nbytes):
    """Contiguous device copy of nbytes (multiple of 16) on the current stream."""
    import torch
    rc = _load().kvmw_plain_copy(dst.data_ptr(), src.data_ptr(), int(nbytes),
                                 torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError("kvmw_plain_copy failed with %d" % rc)


REF_COPY, REF_READ, REF_WRITE = 0, 1, 2


def ref_stream(mode, src, dst, run_bytes, n_runs, src_random, dst_random, sink, src_rot=0, dst_rot=0):
    """One launch of the reference access-pattern kernel (see fill.hip): n_runs runs of
    run_bytes each, read from `src` and / or written to `dst` (torch tensors spanning
    the buffers), at consecutive run slots or at pseudo-randomly permuted slots over
    the largest power-of-two number of slots the buffer holds.  *_rot: workgroup c of
    run r takes 4 KiB chunk (c + (rot & 7) + (rot >> 3) * r) % chunks of that side."""
    import torch

    def bits(buf, random):
        slots = buf.numel() * buf.element_size() // run_bytes
        assert slots >= n_runs
        if not random:
            return 0
        b = slots.bit_length() - 1            # 2^b <= slots
        assert n_runs <= 1 << b
        return b

    rc = _load().kvmw_ref_stream(mode, src.data_ptr() if src is not None else None,
                                 dst.data_ptr() if dst is not None else None, run_bytes, n_runs,
                                 bits(src, src_random) if src is not None else 0,
                                 bits(dst, dst_random) if dst is not None else 0, int(src_rot), int(dst_rot),
                                 sink.data_ptr(), torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError("kvmw_ref_stream failed with %d" % rc)


def ref_walk(src, n_bytes, stride_pieces, n_steps, sliced, sink):
    """One launch of the walking read kernel (see fill.hip): workgroups of four waves that
    each make n_steps steps of four 4 KiB pieces from the lower half of `src` and four from
    the upper half; n_bytes in total (rounded down to whole workgroups).  Returns the bytes read."""
    import torch
    half_pieces = src.numel() * src.element_size() // 8192
    n_wg = n_bytes // (n_steps * 8 * 4096)
    assert n_wg >= 1 and 3 * stride_pieces < half_pieces
    rc = _load().kvmw_ref_walk(src.data_ptr(), half_pieces, int(stride_pieces), int(n_steps), n_wg,
                               1 if sliced else 0, sink.data_ptr(), torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError("kvmw_ref_walk failed with %d" % rc)
    return n_wg * n_steps * 8 * 4096


def fill_pool(mem, model, n_blocks, seed, stream_id, strides=None, b0=0, b1=None):
    """Fill blocks [b0,b1) of a device pool (torch uint8/int16 tensor) in place."""
    import torch
    st = canonical_strides(model, n_blocks) if strides is None else np.asarray(strides)
    st_bytes = np.ascontiguousarray(st * 2, dtype=np.int64)
    b1 = n_blocks if b1 is None else b1
    rc = _load().kvmw_fill_pool(mem.data_ptr(), st_bytes.ctypes.data, model.L, model.H, model.D,
                                model.B, 1 if model.dtype == "bf16" else 0, b0, b1,
                                seed & 0xFFFFFFFF, stream_id,
                                torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError("kvmw_fill_pool failed with %d" % rc)


def gen_blocks(out, ids_dev, model, seed, stream_id, plane):
    """out[i] <- generator content of block ids_dev[i] of `plane` (dense [H][B][D]
    16-bit per block; `out` is a torch tensor of at least len(ids) blocks)."""
    import torch
    n = int(ids_dev.numel())
    assert ids_dev.dtype == torch.int32 and ids_dev.is_contiguous()
    assert out.numel() * out.element_size() >= n * model.H * model.B * model.D * 2
    rc = _load().kvmw_gen_blocks(out.data_ptr(), ids_dev.data_ptr(), n, model.H, model.B, model.D,
                                 1 if model.dtype == "bf16" else 0, seed & 0xFFFFFFFF, stream_id,
                                 plane, torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError("kvmw_gen_blocks failed with %d" % rc)


MIX64_GOLD = 0x9E3779B97F4A7C15


def plane_block_hashes(mem, model, n_blocks):
    """Position-sensitive 64-bit hash of every (plane, block) of a dense canonical
    pool -> int64 tensor [2L, n_blocks]: sum over the block's 8-byte words of
    splitmix64(word + (index + 1) * 0x9E3779B97F4A7C15), mod 2^64.  Used to show that
    blocks were left untouched; unlike a plain sum it sees words that moved."""
    import torch
    st = np.ascontiguousarray(canonical_strides(model, n_blocks)[:3] * 2, dtype=np.int64)
    words = model.H * model.B * model.D * 2 // 8
    out = torch.empty(2 * model.L, n_blocks, dtype=torch.int64, device=mem.device)
    rc = _load().kvmw_block_hashes(mem.data_ptr(), st.ctypes.data, model.L, n_blocks, words,
                                   out.data_ptr(), torch.cuda.current_stream().cuda_stream)
    if rc != 0:
        raise RuntimeError("kvmw_block_hashes failed with %d" % rc)
    return out


def block_hash_host(block_u16):
    """The same hash of one block given as a uint16 array (numpy; for checking the kernel)."""
    w = np.ascontiguousarray(block_u16).reshape(-1).view(np.uint64)
    with np.errstate(over="ignore"):
        z = w + (np.arange(1, len(w) + 1, dtype=np.uint64) * np.uint64(MIX64_GOLD))
        z = (z ^ (z >> np.uint64(30))) * np.uint64(0xBF58476D1CE4E5B9)
        z = (z ^ (z >> np.uint64(27))) * np.uint64(0x94D049BB133111EB)
        z = z ^ (z >> np.uint64(31))
        return int(z.sum(dtype=np.uint64))
