"""Seeded synthetic inputs for the paged-KV migration path.

This module only *generates inputs*: KV / query values, request lengths, block
placements, destination occupancy and migration orders.  It contains none of
the method's arithmetic (no copying between pools, no attention) and is the one
module the CPU oracle's tests and the HIP path's tests both draw from.

The inputs stand in for the workloads of arXiv 2501.06709, Sec. "Experiment":
LLaMA-2 7B / 13B KV shapes (plus a grouped-query 8B shape) and conversation
length distributions of chat datasets scaled for long context, which are
replaced here by seeded log-normal lengths.

Values are produced by a counter-based generator so that any block of a pool
can be regenerated anywhere (numpy here, a HIP fill kernel in ``fill.hip``)
without moving the pool: element (plane p = layer*2+kv, block b, w = (head*B +
slot)*D + dim) of stream `stream` is

    key = mix32(seed ^ mix32(stream * 0x9E3779B9 + p + 1))
    kb  = mix32(key + b * 0x85EBCA6B)
    x   = mix32(kb + w);  y = mix32(x ^ 0x68E31DA4)
    n   = (sum of the 8 bytes of x and y) - 1020          # Irwin-Hall, n = 8
    val = round_to_dtype(float32(n) * float32(1 / 209.0239))

i.e. approximately N(0,1) (exact mean 0, variance 1, support +-4.88), all in
uint32 / one float32 multiply so host and device agree bit for bit.  mix32 is
the public "lowbias32" 32-bit finaliser (xor-shift 16, * 0x7feb352d, xor-shift
15, * 0x846ca68b, xor-shift 16).
"""
from dataclasses import dataclass, field

import numpy as np

_M1 = np.uint32(0x7FEB352D)
_M2 = np.uint32(0x846CA68B)
_GOLD = 0x9E3779B9
_BLK = 0x85EBCA6B
_YX = np.uint32(0x68E31DA4)
INV_SD = np.float32(float.fromhex("0x1.398896p-8"))  # float32(1 / 209.0239)

STREAM_SRC = 1
STREAM_DST = 2
STREAM_Q = 3


def mix32(x):
    x = np.asarray(x, dtype=np.uint32).copy()
    x ^= x >> np.uint32(16)
    x *= _M1
    x ^= x >> np.uint32(15)
    x *= _M2
    x ^= x >> np.uint32(16)
    return x


def _mix32_scalar(v):
    return int(mix32(np.array([v & 0xFFFFFFFF], dtype=np.uint32))[0])


def f32_to_bits16(f, dtype):
    """Round float32 values to fp16 / bf16 (nearest even) and return the bits."""
    f = np.asarray(f, dtype=np.float32)
    if dtype == "f16":
        return f.astype(np.float16).view(np.uint16)
    assert dtype == "bf16"
    u = f.view(np.uint32)
    return ((u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)).astype(
        np.uint16)


def bits16_to_f64(bits, dtype):
    """Exact widening, done with numpy's own conversions (not the oracle's)."""
    bits = np.asarray(bits, dtype=np.uint16)
    if dtype == "f16":
        return bits.view(np.float16).astype(np.float64)
    with np.errstate(invalid="ignore"):
        return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def plane_key(seed, stream, plane):
    return _mix32_scalar(seed ^ _mix32_scalar(stream * _GOLD + plane + 1))


def gen_values(seed, stream, plane, block, w, dtype):
    """16-bit patterns for element indices `w` (array) of one (plane, block)."""
    kb = _mix32_scalar(plane_key(seed, stream, plane) + (int(block) * _BLK))
    with np.errstate(over="ignore"):
        x = mix32(np.uint32(kb) + np.asarray(w, dtype=np.uint32))
        y = mix32(x ^ _YX)
    s = np.zeros(x.shape, dtype=np.int32)
    for sh in (0, 8, 16, 24):
        s += ((x >> np.uint32(sh)) & np.uint32(0xFF)).astype(np.int32)
        s += ((y >> np.uint32(sh)) & np.uint32(0xFF)).astype(np.int32)
    f = (s - 1020).astype(np.float32) * INV_SD
    return f32_to_bits16(f, dtype)


def gen_block(seed, stream, model, plane, block):
    """One (plane, block) of a pool as uint16 [H][B][D]."""
    n = model.H * model.B * model.D
    return gen_values(seed, stream, plane, block, np.arange(n, dtype=np.uint32),
                      model.dtype).reshape(model.H, model.B, model.D)


def gen_blocks(seed, stream, model, plane, blocks):
    """Blocks `blocks` of one plane as uint16 [len(blocks)][H][B][D] (one vectorised
    pass: for regenerating many blocks of a large pool on the host)."""
    blocks = np.asarray(blocks, dtype=np.int64)
    n = model.H * model.B * model.D
    key = plane_key(seed, stream, plane)
    with np.errstate(over="ignore"):
        kb = mix32((np.uint32(key) + (blocks.astype(np.uint64) * _BLK).astype(np.uint32)))
        x = mix32(kb[:, None] + np.arange(n, dtype=np.uint32)[None, :])
        y = mix32(x ^ _YX)
    s = np.zeros(x.shape, dtype=np.int32)
    for sh in (0, 8, 16, 24):
        s += ((x >> np.uint32(sh)) & np.uint32(0xFF)).astype(np.int32)
        s += ((y >> np.uint32(sh)) & np.uint32(0xFF)).astype(np.int32)
    f = (s - 1020).astype(np.float32) * INV_SD
    return f32_to_bits16(f, model.dtype).reshape(len(blocks), model.H, model.B, model.D)


def gen_pool_host(seed, stream, model, n_blocks, strides=None, blocks=None):
    """A whole pool on the host as a flat uint16 array (small pools only).
    `blocks`: only these ids are generated, the rest stays zero."""
    st = canonical_strides(model, n_blocks) if strides is None else np.asarray(strides)
    span = pool_span_elems(model, n_blocks, st)
    pool = np.zeros(span, dtype=np.uint16)
    ids = range(n_blocks) if blocks is None else blocks
    h = np.arange(model.H)[:, None, None] * st[3]
    s = np.arange(model.B)[None, :, None] * st[4]
    d = np.arange(model.D)[None, None, :]
    inner = (h + s + d).astype(np.int64)
    for p in range(2 * model.L):
        base_p = (p // 2) * st[0] + (p % 2) * st[1]
        for b in ids:
            pool[base_p + int(b) * st[2] + inner] = gen_block(seed, stream, model, p, b)
    return pool


def gen_q(seed, model, n_req):
    """Query vectors uint16 [n_req][L][Hq][D]: request r is 'block' r of stream Q."""
    n = model.L * model.Hq * model.D
    out = np.zeros((n_req, n), dtype=np.uint16)
    for r in range(n_req):
        out[r] = gen_values(seed, STREAM_Q, 0, r, np.arange(n, dtype=np.uint32), model.dtype)
    return out.reshape(n_req, model.L, model.Hq, model.D)


@dataclass(frozen=True)
class Model:
    name: str
    L: int
    H: int
    Hq: int
    D: int
    B: int
    dtype: str  # "f16" | "bf16"

    @property
    def bytes_per_token(self):
        return self.L * 2 * self.H * self.D * 2

    @property
    def block_bytes(self):
        return self.B * self.bytes_per_token


TINY = Model("tiny", 2, 4, 4, 64, 16, "f16")
LLAMA2_7B = Model("llama2_7b", 32, 32, 32, 128, 16, "f16")
LLAMA3_8B = Model("llama3_8b_gqa", 32, 8, 32, 128, 16, "bf16")
LLAMA2_13B = Model("llama2_13b", 40, 40, 40, 128, 16, "f16")


def canonical_strides(model, n_blocks):
    slot = model.D
    head = model.B * slot
    block = model.H * head
    kv = n_blocks * block
    return np.array([2 * kv, kv, block, head, slot], dtype=np.int64)


def pool_span_elems(model, n_blocks, st):
    return int((model.L - 1) * st[0] + st[1] + (n_blocks - 1) * st[2] + (model.H - 1) * st[3]
               + (model.B - 1) * st[4] + model.D)


@dataclass
class Workload:
    """One migration batch: which requests move, from which blocks, how far."""
    name: str
    model: Model
    seed: int
    n_blocks_src: int
    n_blocks_dst: int
    lens: np.ndarray            # [n_requests] tokens of every live request
    src_tables: list            # per request: int32 ids covering ceil(len/B) blocks
    migrate_ids: np.ndarray     # indices of the requests that move
    k: np.ndarray               # [len(migrate_ids)] split points
    dst_occupied: np.ndarray    # uint8 [n_blocks_dst], 1 = in use before migration
    notes: list = field(default_factory=list)

    def src_csr(self):
        """CSR tables (offsets, blocks) of the migrated requests, full length."""
        tabs = [self.src_tables[i] for i in self.migrate_ids]
        off = np.zeros(len(tabs) + 1, dtype=np.int32)
        off[1:] = np.cumsum([len(t) for t in tabs])
        blocks = np.concatenate(tabs).astype(np.int32) if tabs else np.zeros(0, np.int32)
        return off, blocks

    def n_dst_blocks(self):
        return [-(-int(k) // self.model.B) for k in self.k]

    def payload_bytes(self):
        return int(np.sum(self.k.astype(np.int64))) * self.model.bytes_per_token


def lognormal_lengths(rng, n, median, sigma, cap):
    z = rng.standard_normal(n)
    v = np.rint(np.exp(np.log(float(median)) + sigma * z))
    return np.clip(v, 1, cap).astype(np.int64)


def _rng(seed):
    return np.random.Generator(np.random.Philox(seed))


def _place(rng, lens, B, n_blocks):
    """Source placement: requests take consecutive runs of a seeded permutation."""
    nb = -(-lens // B)
    if int(nb.sum()) > n_blocks:
        raise ValueError("source pool of %d blocks cannot hold %d" % (n_blocks, int(nb.sum())))
    perm = rng.permutation(n_blocks).astype(np.int32)
    tabs, p = [], 0
    for n in nb:
        tabs.append(perm[p:p + int(n)].copy())
        p += int(n)
    return tabs


def _fit_requests(lens, B, n_blocks, n_keep_min):
    """Drop trailing requests until the live set fits the source pool."""
    nb = -(-lens // B)
    n = len(lens)
    while n > n_keep_min and int(nb[:n].sum()) > n_blocks:
        n -= 1
    return lens[:n]


CONFIG_NAMES = ("tiny", "llama2_7b", "llama3_8b_gqa", "llama2_13b_long")


def make(name, n_blocks_src=None, n_blocks_dst=None, n_requests=None, n_migrate=None,
         len_cap=None, seed=None):
    """Build one of the benchmark workloads; the keyword overrides shrink it for
    cases the CPU oracle has to finish in seconds (shape and structure stay)."""
    idx = CONFIG_NAMES.index(name)
    seed = 20250106 + idx if seed is None else seed
    rng = _rng(seed)
    notes = []
    if name == "tiny":
        model, nbs, nbd, nreq, nmig = TINY, 1024, 1024, 8, 4
        nreq, nmig = n_requests or nreq, n_migrate or nmig
        lens = rng.integers(1, (len_cap or 256) + 1, size=nreq).astype(np.int64)
        kfrac, occ = 1.0, 0.0
    elif name == "llama2_7b":
        model, nbs, nbd, nreq, nmig = LLAMA2_7B, 16384, 16384, 64, 8
        nreq, nmig = n_requests or nreq, n_migrate or nmig
        lens = lognormal_lengths(rng, nreq, 512, 0.8, len_cap or 4096)
        kfrac, occ = 1.0, 0.0
    elif name == "llama3_8b_gqa":
        model, nbs, nbd, nreq, nmig = LLAMA3_8B, 65536, 65536, 256, 32
        nreq, nmig = n_requests or nreq, n_migrate or nmig
        lens = lognormal_lengths(rng, nreq, 1024, 0.8, len_cap or 8192)
        kfrac, occ = 0.75, 0.5
    else:
        # The nominal 40000-block 13B pool is 488 GiB and cannot exist in 288 GB
        # of HBM; the pools are capped while layout, request sizes, random source
        # placement and 30 % destination occupancy are kept.
        model, nbs, nbd, nreq, nmig = LLAMA2_13B, 8704, 12288, 4, 4
        nreq, nmig = n_requests or nreq, n_migrate or nmig
        lens = np.full(nreq, len_cap or 32768, dtype=np.int64)
        kfrac, occ = 1.0, 0.3
        notes.append("source pool capped from the nominal 40000 blocks to fit HBM")
    nbs = n_blocks_src or nbs
    nbd = n_blocks_dst or nbd
    fitted = _fit_requests(lens, model.B, nbs, nmig)
    if len(fitted) < len(lens):
        notes.append("live requests reduced from %d to %d to fit the source pool"
                     % (len(lens), len(fitted)))
        lens = fitted
    tabs = _place(rng, lens, model.B, nbs)
    migrate_ids = np.arange(min(nmig, len(lens)), dtype=np.int64)
    k = np.floor(kfrac * lens[migrate_ids]).astype(np.int32) if kfrac < 1.0 else \
        lens[migrate_ids].astype(np.int32)
    occupied = (rng.random(nbd) < occ).astype(np.uint8) if occ > 0 else np.zeros(nbd, np.uint8)
    need = sum(-(-int(x) // model.B) for x in k)
    if int((occupied == 0).sum()) < need:
        raise ValueError("destination pool has %d free blocks, %d needed"
                         % (int((occupied == 0).sum()), need))
    return Workload(name, model, seed, nbs, nbd, lens, tabs, migrate_ids, k, occupied, notes)
