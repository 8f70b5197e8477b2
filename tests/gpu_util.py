"""Helpers shared by the GPU parity tests: build a case on host and device."""
import numpy as np
import torch

import kvm_workload as wl
import paper_2501_06709_amd as kvm

DEV = "cuda:0"


def csr(tables):
    off = np.zeros(len(tables) + 1, dtype=np.int32)
    off[1:] = np.cumsum([len(t) for t in tables])
    blk = np.concatenate(tables).astype(np.int32) if len(tables) and off[-1] else np.zeros(0, np.int32)
    return off, blk


def layout_for(m, n_blocks, strides=None):
    lay = kvm.kvm_layout_canonical(m.L, m.H, m.Hq, m.D, m.B, m.dtype, n_blocks)
    if strides is not None:
        (lay.stride_layer, lay.stride_kv, lay.stride_block, lay.stride_head,
         lay.stride_slot) = (int(s) for s in strides)
    return lay


def to_dev(host_u16):
    return torch.from_numpy(host_u16.view(np.int16)).to(DEV)


def to_host(t):
    return t.cpu().numpy().view(np.uint16).reshape(-1)


def dev_table(blk):
    # at least one element so that the pointer is never NULL
    return torch.from_numpy(np.concatenate([blk, np.zeros(1, np.int32)])).to(DEV)


class Side:
    """One pool on host (uint16 array) and device, with its tables."""

    def __init__(self, m, n_blocks, host, tables, k, strides=None, host_ids=True, start=None):
        self.m, self.n_blocks = m, n_blocks
        self.st = np.asarray(wl.canonical_strides(m, n_blocks) if strides is None else strides,
                             dtype=np.int64)
        self.host = host
        self.dev = to_dev(host)
        self.layout = layout_for(m, n_blocks, self.st)
        self.pool = kvm.Pool(self.dev, n_blocks, self.layout)
        self.tables = tables
        self.off, self.blk = csr(tables)
        self.k = np.asarray(k, dtype=np.int32)
        self.blk_dev = dev_table(self.blk)
        self.start = None if start is None else np.asarray(start, dtype=np.int32)
        self.batch = kvm.Batch(self.off, self.blk, self.k, self.blk_dev, host_ids=host_ids,
                               start=self.start)


def random_bits(rng, n):
    """Arbitrary 16-bit patterns (NaNs, infinities, negative zero included)."""
    return rng.integers(0, 65536, size=n, dtype=np.uint16)


def tables_from_perm(rng, n_blocks, counts):
    perm = rng.permutation(n_blocks).astype(np.int32)
    assert sum(counts) <= n_blocks
    tabs, p = [], 0
    for n in counts:
        tabs.append(perm[p:p + n].copy())
        p += n
    return tabs


def make_pair(m, n_src, n_dst, lens, ks, seed, src_strides=None, dst_strides=None, finite=False,
              host_ids=True, start=None):
    """Source and destination sides of a migration with random placement."""
    rng = np.random.default_rng(seed)
    B = m.B
    s_tabs = tables_from_perm(rng, n_src, [-(-ln // B) for ln in lens])
    d_tabs = tables_from_perm(rng, n_dst, [-(-k // B) for k in ks])
    st_s = wl.canonical_strides(m, n_src) if src_strides is None else np.asarray(src_strides)
    st_d = wl.canonical_strides(m, n_dst) if dst_strides is None else np.asarray(dst_strides)
    if finite:
        h_src = wl.gen_pool_host(seed, wl.STREAM_SRC, m, n_src, st_s)
        h_dst = wl.gen_pool_host(seed, wl.STREAM_DST, m, n_dst, st_d)
    else:
        h_src = random_bits(rng, wl.pool_span_elems(m, n_src, st_s))
        h_dst = random_bits(rng, wl.pool_span_elems(m, n_dst, st_d))
    src = Side(m, n_src, h_src, s_tabs, ks, st_s, host_ids, start)
    dst = Side(m, n_dst, h_dst, d_tabs, ks, st_d, host_ids, start)
    return src, dst


def oracle_migrate(orc, src, dst):
    """Expected destination pool after migrating src -> dst (host copy returned)."""
    m = src.m
    exp = dst.host.copy()
    orc.migrate(src.host, src.st, exp, dst.st, m.L, m.H, m.D, m.B, src.off, src.blk, dst.off,
                dst.blk, src.k, start=src.start)
    return exp


# ---- checks for pools too large for the host ----------------------------------
# The pools are filled by the counter-based generator, whose device kernel and numpy
# form agree bit for bit (tested on whole small pools).  What a block must hold after
# a migration then follows from the definition at block granularity: destination
# block bt_dst[j] of a request holds what the generator gives for its source block
# bt_src[j].  That is compared for EVERY written block on the device; blocks that are
# only partly written, and samples of the others, go to the host and through the
# CPU oracle.

def planes_view(mem, m, n_blocks):
    """A dense canonical pool as int16 [2L][n_blocks][H*B*D]."""
    return mem.view(torch.int16).view(2 * m.L, n_blocks, m.H * m.B * m.D)


def assert_blocks_equal_generator(mem, m, n_blocks, ids, gen_ids, seed, stream, what, chunk_bytes=1 << 30):
    """Every block ids[i] of the pool, in every plane, holds the generator's content
    of block gen_ids[i] of `stream` (all on the device, in chunks)."""
    from kvm_workload import device as wl_device
    ids = np.asarray(ids, dtype=np.int64)
    gen_ids = np.asarray(gen_ids, dtype=np.int32)
    assert len(ids) == len(gen_ids)
    if len(ids) == 0:
        return
    pv = planes_view(mem, m, n_blocks)
    run = m.H * m.B * m.D
    per = max(1, chunk_bytes // (run * 2))
    exp = torch.empty(min(per, len(ids)) * run, dtype=torch.int16, device=mem.device)
    for c in range(0, len(ids), per):
        idx = torch.from_numpy(ids[c:c + per]).to(mem.device)
        gid = torch.from_numpy(np.ascontiguousarray(gen_ids[c:c + per])).to(mem.device)
        n = len(idx)
        for p in range(2 * m.L):
            wl_device.gen_blocks(exp, gid, m, seed, stream, p)
            got = pv[p].index_select(0, idx)
            if not torch.equal(got, exp[:n * run].view(n, run)):
                bad = (got != exp[:n * run].view(n, run)).any(dim=1).nonzero().flatten()[:5].cpu().numpy()
                raise AssertionError("%s: plane %d, blocks %s differ from the generator's blocks %s"
                                     % (what, p, ids[c:c + per][bad], gen_ids[c:c + per][bad]))


def full_and_partial(off, blk, k, B):
    """Splits the blocks that hold tokens [0,k[r]) into completely written ones
    (positions into blk) and, per request, the partly written last one."""
    full, partial = [], []
    for r in range(len(k)):
        nfull = int(k[r]) // B
        full.append(np.arange(off[r], off[r] + nfull))
        if int(k[r]) % B:
            partial.append((r, nfull, int(k[r]) % B))
    return (np.concatenate(full) if full else np.zeros(0, np.int64)), partial
