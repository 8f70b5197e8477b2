"""TEST INFRASTRUCTURE, not product code: Python face of the CPU oracle.

Wraps ``kvm_oracle.c`` (compiled with gcc by :func:`build`) and adds the
integer-only host steps of the path (free-list allocation, source release)
in plain Python.  Only ``tests/``, the smoke check and the benchmark's
``cpu_baseline`` leg may import this module; it imports nothing from the HIP
package.

Paper passages followed (arXiv 2501.06709): Sec. "Background & Related Work"
(paged, non-contiguous KV cache), Sec. "Motivation" Finding 4 and Sec.
"Adaptive Request Migration" / "Hybrid Migration" (a request moves either as KV
cache or as tokens), "Boundary Profiling" (source memory is released only after
the transfer), Sec. "System Model" (KV bytes linear in tokens, capacity
constraint Eq. 2).
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvm_oracle.c")
_LIB = os.path.join(_HERE, "libkvm_oracle.so")
_lib = None


def build(force=False):
    """Compile the C oracle with gcc (-O2, no fast-math: fp64 stays IEEE)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-std=c99", "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"])
    return _LIB


_I32P = np.ctypeslib.ndpointer(dtype=np.int32, flags="C_CONTIGUOUS")
_I64P = np.ctypeslib.ndpointer(dtype=np.int64, flags="C_CONTIGUOUS")
_U16P = np.ctypeslib.ndpointer(dtype=np.uint16, flags="C_CONTIGUOUS")
_F64P = np.ctypeslib.ndpointer(dtype=np.float64, flags="C_CONTIGUOUS")
_INT = ctypes.c_int


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.orc_bytes_per_token.restype = ctypes.c_int64
        lib.orc_bytes_per_token.argtypes = [_INT, _INT, _INT]
        lib.orc_migrate.restype = None
        lib.orc_migrate.argtypes = [_U16P, _I64P, _U16P, _I64P, _INT, _INT, _INT, _INT, _INT,
                                    _I32P, _I32P, _I32P, _I32P, _I32P, _I32P, _INT, _INT]
        lib.orc_pack.restype = None
        lib.orc_pack.argtypes = [_U16P, _I64P, _U16P, _INT, _INT, _INT, _INT, _INT,
                                 _I32P, _I32P, _I32P, _I32P, _INT, _INT]
        lib.orc_unpack.restype = None
        lib.orc_unpack.argtypes = [_U16P, _U16P, _I64P, _INT, _INT, _INT, _INT, _INT,
                                   _I32P, _I32P, _I32P, _I32P, _INT, _INT]
        lib.orc_widen.restype = ctypes.c_double
        lib.orc_widen.argtypes = [ctypes.c_uint16, _INT]
        lib.orc_paged_decode.restype = None
        lib.orc_paged_decode.argtypes = [_U16P, _I64P, _INT, _INT, _INT, _INT, _INT, _INT, _INT,
                                         _I32P, _I32P, _I32P, _U16P, _F64P, ctypes.c_double]
        _lib = lib
    return _lib


DTYPE_CODE = {"f16": 0, "bf16": 1}


def bytes_per_token(L, H, D):
    """KV bytes of one token: layers x {K,V} x KV heads x head_dim x 2 bytes."""
    return int(_load().orc_bytes_per_token(L, H, D))


def canonical_strides(L, H, D, B, n_blocks):
    """Element strides (layer, kv, block, head, slot) of the dense layout
    pool[layer][kv][block][head][slot][dim]."""
    slot = D
    head = B * slot
    block = H * head
    kv = n_blocks * block
    layer = 2 * kv
    return np.array([layer, kv, block, head, slot], dtype=np.int64)


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _st(a):
    a = np.ascontiguousarray(np.asarray(a, dtype=np.int64))
    assert a.shape == (5,)
    return a


def _check_tables(pool_elems, st, L, H, D, B, off, blocks, k):
    """Bounds check so that a bad test input raises instead of corrupting memory."""
    off, blocks, k = np.asarray(off), np.asarray(blocks), np.asarray(k)
    assert off[0] == 0 and off[-1] <= len(blocks) and len(k) == len(off) - 1
    for r in range(len(k)):
        nb = int(off[r + 1] - off[r])
        assert 0 <= k[r] <= nb * B, (r, int(k[r]), nb)
        used = blocks[off[r]: off[r] + -(-int(k[r]) // B)]
        if len(used):
            assert used.min() >= 0
            top = ((L - 1) * st[0] + st[1] + int(used.max()) * st[2] + (H - 1) * st[3]
                   + (B - 1) * st[4] + D - 1)
            assert top < pool_elems, "block id beyond pool"


def _start(start, k):
    st = np.zeros(len(k), dtype=np.int32) if start is None else _i32(start)
    assert len(st) == len(k) and (st >= 0).all() and (st <= k).all()
    return st


def migrate(src, src_st, dst, dst_st, L, H, D, B, src_off, src_blocks, dst_off, dst_blocks, k,
            layers=None, start=None):
    """dst <- tokens [start[r],k[r]) of every request (start defaults to 0), in
    place; src is not written."""
    src_off, src_blocks = _i32(src_off), _i32(src_blocks)
    dst_off, dst_blocks, k = _i32(dst_off), _i32(dst_blocks), _i32(k)
    src_st, dst_st = _st(src_st), _st(dst_st)
    _check_tables(src.size, src_st, L, H, D, B, src_off, src_blocks, k)
    _check_tables(dst.size, dst_st, L, H, D, B, dst_off, dst_blocks, k)
    lb, le = layers if layers is not None else (0, L)
    _load().orc_migrate(src, src_st, dst, dst_st, L, H, D, B, len(k), src_off, src_blocks,
                        dst_off, dst_blocks, k, _start(start, k), lb, le)


def staging_elems(L, H, D, k, start=None):
    n = np.asarray(k, dtype=np.int64) - (0 if start is None else np.asarray(start, dtype=np.int64))
    return int(np.sum(n)) * L * 2 * H * D


def pack(src, src_st, L, H, D, B, off, blocks, k, stage=None, layers=None, start=None):
    """Returns the staging buffer (uint16) of tokens [start[r],k[r]) of every request."""
    off, blocks, k, src_st = _i32(off), _i32(blocks), _i32(k), _st(src_st)
    _check_tables(src.size, src_st, L, H, D, B, off, blocks, k)
    st = _start(start, k)
    if stage is None:
        stage = np.zeros(staging_elems(L, H, D, k, st), dtype=np.uint16)
    assert stage.size >= staging_elems(L, H, D, k, st)
    lb, le = layers if layers is not None else (0, L)
    _load().orc_pack(src, src_st, stage, L, H, D, B, len(k), off, blocks, k, st, lb, le)
    return stage


def unpack(stage, dst, dst_st, L, H, D, B, off, blocks, k, layers=None, start=None):
    """Scatter a staging buffer into dst's blocks, in place."""
    off, blocks, k, dst_st = _i32(off), _i32(blocks), _i32(k), _st(dst_st)
    _check_tables(dst.size, dst_st, L, H, D, B, off, blocks, k)
    st = _start(start, k)
    assert stage.size >= staging_elems(L, H, D, k, st)
    lb, le = layers if layers is not None else (0, L)
    _load().orc_unpack(stage, dst, dst_st, L, H, D, B, len(k), off, blocks, k, st, lb, le)


def widen(bits, dtype):
    """Exact value of a 16-bit float pattern as a Python float."""
    return float(_load().orc_widen(int(bits), DTYPE_CODE[dtype]))


def paged_decode(pool, st, L, H, Hq, D, B, dtype, off, blocks, k, q, scale=None, out=None):
    """fp64 attention of one query per (request, layer, query head) over tokens
    [0,k[r]); q is uint16 [n_req, L, Hq, D]; returns float64 of the same shape."""
    off, blocks, k, st = _i32(off), _i32(blocks), _i32(k), _st(st)
    _check_tables(pool.size, st, L, H, D, B, off, blocks, k)
    assert Hq % H == 0
    q = np.ascontiguousarray(q, dtype=np.uint16)
    assert q.shape == (len(k), L, Hq, D)
    if out is None:
        out = np.zeros(q.shape, dtype=np.float64)
    if scale is None:
        scale = 1.0 / np.sqrt(float(D))
    _load().orc_paged_decode(pool, st, L, H, Hq, D, B, DTYPE_CODE[dtype], len(k), off, blocks, k,
                             q, out, float(scale))
    return out


class FreeList:
    """Destination-side block allocator of the oracle: lowest free id first,
    all-or-nothing (capacity constraint of Sec. "System Model", Eq. 2)."""

    def __init__(self, n_blocks, occupied=None):
        self.n_blocks = int(n_blocks)
        self.free = [True] * self.n_blocks
        if occupied is not None:
            for b in range(self.n_blocks):
                if occupied[b]:
                    self.free[b] = False

    def available(self):
        return sum(self.free)

    def alloc(self, n):
        """Returns the n lowest free ids (ascending) or None when fewer are free."""
        ids = []
        for b in range(self.n_blocks):
            if len(ids) == n:
                break
            if self.free[b]:
                ids.append(b)
        if len(ids) < n:
            return None
        for b in ids:
            self.free[b] = False
        return ids

    def release(self, ids):
        """Source release after a completed transfer; rejects bad or repeated ids."""
        ids = [int(b) for b in ids]
        if len(set(ids)) != len(ids):
            raise ValueError("repeated id")
        for b in ids:
            if not 0 <= b < self.n_blocks or self.free[b]:
                raise ValueError("id %d not allocated" % b)
        for b in ids:
            self.free[b] = True


CLASS_KV, CLASS_TOKENS, CLASS_DEFER = 0, 1, 2


def divide_moves(moves, comm_boundary, comp_boundary, policy="first_fit"):
    """Hybrid-migration divider (Sec. "Adaptive Request Migration", "Hybrid
    Migration" / "Global Consensus"): each pending move, in list order, goes to the
    KV-transfer class if its bytes still fit the link's communication boundary, to
    the token-transfer class if its tokens still fit the destination's computation
    boundary, else it is deferred.  `moves`: (link, dst, kv_bytes, tokens).
    first_fit tries KV first; best_fit takes the class whose bin keeps the smaller
    free fraction of its boundary (a bin with boundary 0 counts as fraction 0; ties
    go to KV).  Returns the list of classes."""
    from fractions import Fraction
    link_left = [int(c) for c in comm_boundary]
    inst_left = [int(c) for c in comp_boundary]
    out = []
    for link, dst, kv_bytes, tokens in moves:
        fits_kv = kv_bytes <= link_left[link]
        fits_tok = tokens <= inst_left[dst]
        if fits_kv and fits_tok and policy == "best_fit":
            f_kv = Fraction(link_left[link] - kv_bytes, comm_boundary[link]) if comm_boundary[link] else 0
            f_tok = Fraction(inst_left[dst] - tokens, comp_boundary[dst]) if comp_boundary[dst] else 0
            cls = CLASS_KV if f_kv <= f_tok else CLASS_TOKENS
        elif fits_kv:
            cls = CLASS_KV
        elif fits_tok:
            cls = CLASS_TOKENS
        else:
            cls = CLASS_DEFER
        if cls == CLASS_KV:
            link_left[link] -= kv_bytes
        elif cls == CLASS_TOKENS:
            inst_left[dst] -= tokens
        out.append(cls)
    return out
