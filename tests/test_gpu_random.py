"""Seeded random sweep of the three copy paths against the oracle: shapes, strides,
split points, token ranges and launch options drawn together, small pools, one
process.  The fixed cases elsewhere pin what each feature must do; this looks for
index arithmetic that only fails in combination."""
import numpy as np
import pytest
import torch

import kvm_workload as wl
import paper_2501_06709_amd as kvm

from gpu_util import Side, make_pair
from test_gpu_decode import gpu_decode, oracle_decode
from test_gpu_parity import run_all_three

pytestmark = pytest.mark.gpu

OPTIONS = ("copy.order", "copy.stage_linear", "copy.nontemporal")


def strides_for(rng, m, n_blocks):
    """Canonical, token-major inside the block, padded rows, or block-major pool."""
    kind = int(rng.integers(4))
    if kind == 0:
        return None
    if kind == 1:   # [layer][kv][block][slot][head][dim]
        slot = m.H * m.D
        return np.array([2 * n_blocks * m.B * slot, n_blocks * m.B * slot, m.B * slot, m.D, slot], np.int64)
    if kind == 2:   # canonical order with 8 elements of padding after every token row
        row = m.D + 8
        head = m.B * row
        blk = m.H * head
        return np.array([2 * n_blocks * blk, n_blocks * blk, blk, head, row], np.int64)
    blk = m.H * m.B * m.D   # [block][layer][kv][head][slot][dim]
    return np.array([2 * blk, blk, 2 * m.L * blk, m.B * m.D, m.D], np.int64)


@pytest.mark.parametrize("seed", range(48))
def test_random_case(oracle, seed):
    rng = np.random.default_rng(1000 + seed)
    m = wl.Model("r%d" % seed, int(rng.integers(1, 4)), int(rng.integers(1, 5)), 0,
                 int(rng.choice([64, 80, 128, 256])), int(rng.choice([8, 12, 16, 32])),
                 str(rng.choice(["f16", "bf16"])))
    m = wl.Model(m.name, m.L, m.H, m.H, m.D, m.B, m.dtype)
    n_req = int(rng.integers(1, 7))
    lens = [int(rng.integers(1, 6 * m.B)) for _ in range(n_req)]
    ks = [int(rng.integers(0, ln + 1)) if rng.random() < 0.7 else ln for ln in lens]
    if rng.random() < 0.5:
        start = None
    elif rng.random() < 0.5:
        start = [int(rng.integers(0, k // m.B + 1)) * m.B if k else 0 for k in ks]   # block-aligned ranges
        start = [min(s, k) for s, k in zip(start, ks)]
    else:
        start = [int(rng.integers(0, k + 1)) for k in ks]
    n_src = sum(-(-ln // m.B) for ln in lens) + int(rng.integers(0, 9))
    n_dst = sum(-(-k // m.B) for k in ks) + int(rng.integers(1, 9))
    values = [int(rng.integers(2)), int(rng.integers(4)), int(rng.random() < 0.8)]
    try:
        for name, v in zip(OPTIONS, values):
            kvm.kvm_set_option(name, v)
        src, dst = make_pair(m, n_src, n_dst, lens, ks, seed=2000 + seed, src_strides=strides_for(rng, m, n_src),
                             dst_strides=strides_for(rng, m, n_dst), start=start)
        run_all_three(oracle, src, dst)
    finally:
        kvm.kvm_set_option("reset", 0)
    torch.cuda.synchronize()


DEC_OPTIONS = ("decode.mfma", "decode.cap_waves", "decode.force_splits")


@pytest.mark.parametrize("seed", range(32))
def test_random_decode_case(oracle, seed):
    """Paged decode against the fp64 oracle: tuned and fallback shapes, every group
    size, kernel variant, occupancy instance and split count drawn together."""
    rng = np.random.default_rng(3000 + seed)
    H = int(rng.integers(1, 4))
    G = int(rng.choice([1, 2, 3, 4, 8]))
    D, B = (int(rng.choice([64, 128])), 16) if rng.random() < 0.75 else (int(rng.choice([80, 256])), int(rng.choice([8, 32])))
    m = wl.Model("d%d" % seed, int(rng.integers(1, 3)), H, H * G, D, B, str(rng.choice(["f16", "bf16"])))
    n_req = int(rng.integers(1, 5))
    lens = [int(rng.integers(1, 40 * B)) if rng.random() < 0.8 else int(rng.integers(1, B + 2)) for _ in range(n_req)]
    n_blocks = sum(-(-ln // B) for ln in lens) + 5
    values = [int(rng.integers(-1, 2)), int(rng.integers(-1, 2)), int(rng.choice([0, 0, 1, 2, 5]))]
    try:
        for name, v in zip(DEC_OPTIONS, values):
            kvm.kvm_set_option(name, v)
        src, _ = make_pair(m, n_blocks, 4, lens, [0] * n_req, seed=4000 + seed, finite=True)
        side = Side(m, n_blocks, src.host, src.tables, lens)
        q = wl.gen_q(4000 + seed, m, n_req)
        got = gpu_decode(side, q)
    finally:
        kvm.kvm_set_option("reset", 0)
    ref = oracle_decode(oracle, side, q)
    assert np.abs(got - ref).max() < 2e-3, (m, lens, values, np.abs(got - ref).max())
