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


def plane_block_checksums(mem, model, n_blocks):
    """Wrapping int64 sum of every (plane, block) of a dense pool -> [2L, n_blocks]
    (torch reduction; used to show that blocks were left untouched)."""
    import torch
    words = model.H * model.B * model.D * 2 // 8
    v = mem.view(torch.int64).view(2 * model.L, n_blocks, words)
    out = torch.empty(2 * model.L, n_blocks, dtype=torch.int64, device=mem.device)
    step = max(1, (1 << 28) // (n_blocks * words))  # planes per reduction call
    for p in range(0, 2 * model.L, step):
        out[p:p + step] = v[p:p + step].sum(dim=-1)
    return out
