"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py
times (library defaults), for the 7B-, 8B-GQA- and 13B-shaped configs.

Whole pools (128 GiB and more) cannot be compared on the host, so the checks are:
  * properties that hold at any size: per-(plane, block) checksums of every block
    the migration must not touch are unchanged, the source pool is unchanged, and
    exactly the allocated destination blocks changed;
  * sampled destination blocks (partial last blocks included) compared bit for bit
    with the CPU oracle run on those blocks, regenerated on the host from the
    counter-based generator;
  * sampled decode outputs (request, layer, query head) within 2e-3 of the fp64
    oracle over the regenerated K/V rows.
"""
import numpy as np
import pytest
import torch

import kvm_workload as wl
import paper_2501_06709_amd as kvm
from kvm_workload import device as wl_device

from gpu_util import DEV

pytestmark = pytest.mark.gpu
TOL = 2e-3


def setup(name):
    w = wl.make(name)
    m = w.model
    free_b, _ = torch.cuda.mem_get_info()
    need = (w.n_blocks_src + w.n_blocks_dst) * m.block_bytes
    if need + (12 << 30) > free_b:
        pytest.skip("needs %.0f GiB of HBM, %.0f free" % (need / 2**30, free_b / 2**30))
    lay_s = kvm.kvm_layout_canonical(m.L, m.H, m.Hq, m.D, m.B, m.dtype, w.n_blocks_src)
    lay_d = kvm.kvm_layout_canonical(m.L, m.H, m.Hq, m.D, m.B, m.dtype, w.n_blocks_dst)
    src = torch.empty(kvm.kvm_pool_span_bytes(lay_s, w.n_blocks_src), dtype=torch.uint8, device=DEV)
    dst = torch.empty(kvm.kvm_pool_span_bytes(lay_d, w.n_blocks_dst), dtype=torch.uint8, device=DEV)
    wl_device.fill_pool(src, m, w.n_blocks_src, w.seed, wl.STREAM_SRC)
    wl_device.fill_pool(dst, m, w.n_blocks_dst, w.seed, wl.STREAM_DST)
    fl = kvm.FreeList(w.n_blocks_dst, w.dst_occupied)
    nbk = w.n_dst_blocks()
    ids = fl.alloc(sum(nbk))
    d_off = np.zeros(len(nbk) + 1, np.int32)
    d_off[1:] = np.cumsum(nbk)
    s_off, s_blk = w.src_csr()
    sb = kvm.Batch(s_off, s_blk, w.k, torch.from_numpy(s_blk).to(DEV))
    db = kvm.Batch(d_off, ids, w.k, torch.from_numpy(ids).to(DEV))
    return (w, m, src, dst, kvm.Pool(src, w.n_blocks_src, lay_s), kvm.Pool(dst, w.n_blocks_dst, lay_d),
            sb, db, lay_s)


def sampled_block_check(oracle, w, m, src, dst, sb, db, rng, n_samples):
    run = m.H * m.B * m.D
    sp = src.view(torch.int16).view(2 * m.L, w.n_blocks_src, run)
    dp = dst.view(torch.int16).view(2 * m.L, w.n_blocks_dst, run)
    st1 = oracle.canonical_strides(m.L, m.H, m.D, m.B, 1)
    reqs = [r for r in range(sb.n_req) if w.k[r] > 0]
    picks = [(r, -(-int(w.k[r]) // m.B) - 1) for r in reqs[:3]]          # partial last blocks
    picks += [(int(r), int(rng.integers(-(-int(w.k[r]) // m.B)))) for r in rng.choice(reqs, n_samples)]
    for r, j in picks:
        ns = min(m.B, int(w.k[r]) - j * m.B)
        sblk = int(sb.blocks[sb.offsets[r] + j])
        dblk = int(db.blocks[db.offsets[r] + j])
        mini_src = np.stack([wl.gen_block(w.seed, wl.STREAM_SRC, m, p, sblk) for p in range(2 * m.L)])
        mini_dst = np.stack([wl.gen_block(w.seed, wl.STREAM_DST, m, p, dblk) for p in range(2 * m.L)])
        got_src = sp[:, sblk].cpu().numpy().view(np.uint16).reshape(mini_src.shape)
        assert np.array_equal(got_src, mini_src), "source block %d changed" % sblk
        exp = mini_dst.reshape(-1).copy()
        oracle.migrate(mini_src.reshape(-1), st1, exp, st1, m.L, m.H, m.D, m.B, [0, 1], [0], [0, 1],
                       [0], [ns])
        got = dp[:, dblk].cpu().numpy().view(np.uint16).reshape(-1)
        assert np.array_equal(got, exp), "request %d block %d (-> %d, %d slots) differs" % (r, j, dblk, ns)


def sampled_decode_check(oracle, w, m, sb, out, q, rng, n_samples, reqs=None):
    reqs = [r for r in (reqs if reqs is not None else range(sb.n_req)) if w.k[r] > 0]
    g_size = m.Hq // m.H
    worst = 0.0
    for _ in range(n_samples):
        r = int(rng.choice(reqs))
        l, hq = int(rng.integers(m.L)), int(rng.integers(m.Hq))
        g = hq // g_size
        k = int(w.k[r])
        nb = -(-k // m.B)
        wsel = (g * m.B * m.D + np.arange(m.B * m.D)).astype(np.uint32)
        kv = np.zeros((2, nb, m.B * m.D), dtype=np.uint16)
        for j in range(nb):
            blk = int(sb.blocks[sb.offsets[r] + j])      # the moved bytes are the source's
            for c in range(2):
                kv[c, j] = wl.gen_values(w.seed, wl.STREAM_SRC, 2 * l + c, blk, wsel, m.dtype)
        st = oracle.canonical_strides(1, 1, m.D, m.B, nb)
        ref = oracle.paged_decode(kv.reshape(-1), st, 1, 1, 1, m.D, m.B, m.dtype, [0, nb],
                                  np.arange(nb), [k], q[r, l, hq].reshape(1, 1, 1, m.D))
        err = float(np.abs(out[r, l, hq].astype(np.float64) - ref[0, 0, 0]).max())
        worst = max(worst, err)
        assert err < TOL, "decode (r=%d, l=%d, hq=%d, k=%d): %g" % (r, l, hq, k, err)
    return worst


def run_config(oracle, name, n_block_samples, n_decode_samples, stage_requests):
    w, m, src, dst, ps, pd, sb, db, lay = setup(name)
    rng = np.random.default_rng(7)
    src_sum = wl_device.plane_block_checksums(src, m, w.n_blocks_src)
    dst_sum = wl_device.plane_block_checksums(dst, m, w.n_blocks_dst)

    kvm.kvm_migrate(ps, sb, pd, db)
    torch.cuda.synchronize()
    assert torch.equal(wl_device.plane_block_checksums(src, m, w.n_blocks_src), src_sum), \
        "source pool changed"
    after = wl_device.plane_block_checksums(dst, m, w.n_blocks_dst)
    changed = (after != dst_sum).any(dim=0).cpu().numpy()
    written = np.zeros(w.n_blocks_dst, bool)
    written[db.blocks] = True
    assert not (changed & ~written).any(), "a block outside the destination table changed"
    assert changed[written].all(), "an allocated destination block did not change"
    sampled_block_check(oracle, w, m, src, dst, sb, db, rng, n_block_samples)

    # staged path into a re-filled destination: same end state, sampled
    sel = list(range(min(stage_requests, sb.n_req)))
    k2 = np.zeros_like(w.k)
    k2[sel] = w.k[sel]
    if name == "llama2_13b_long":
        k2[sel] = 8192          # one 13B request prefix: 6.25 GiB of staging
    sb2 = kvm.Batch(sb.offsets, sb.blocks, k2, sb.blocks_dev)
    db2 = kvm.Batch(db.offsets, db.blocks, k2, db.blocks_dev)
    wl_device.fill_pool(dst, m, w.n_blocks_dst, w.seed, wl.STREAM_DST)
    n_stage = kvm.kvm_staging_bytes(lay, sb2)
    stage = torch.empty(n_stage, dtype=torch.uint8, device=DEV)
    kvm.kvm_pack(ps, sb2, stage)
    kvm.kvm_unpack(stage, pd, db2)
    torch.cuda.synchronize()
    del stage
    w2 = wl.Workload(w.name, m, w.seed, w.n_blocks_src, w.n_blocks_dst, w.lens, w.src_tables,
                     w.migrate_ids, k2, w.dst_occupied)
    sampled_block_check(oracle, w2, m, src, dst, sb2, db2, rng, max(2, n_block_samples // 2))
    assert torch.equal(wl_device.plane_block_checksums(src, m, w.n_blocks_src), src_sum)

    # decode over the destination after a full fused migration
    kvm.kvm_migrate(ps, sb, pd, db)
    q = wl.gen_q(w.seed, m, sb.n_req)
    q_dev = torch.from_numpy(q.view(np.int16)).to(DEV)
    out = torch.zeros(q.shape, dtype=torch.float32, device=DEV)
    nws = kvm.kvm_decode_workspace_bytes(lay, db)
    ws = torch.empty(max(nws, 16), dtype=torch.uint8, device=DEV)
    kvm.kvm_paged_decode(pd, db, q_dev, out, workspace=ws, workspace_bytes=nws)
    out_src = torch.zeros_like(out)
    kvm.kvm_paged_decode(ps, sb, q_dev, out_src, workspace=ws, workspace_bytes=nws)
    torch.cuda.synchronize()
    assert torch.equal(out, out_src), "decode over the destination differs from decode over the source"
    worst = sampled_decode_check(oracle, w, m, sb, out.cpu().numpy(), q, rng, n_decode_samples)
    print("%s: %d blocks moved, worst sampled decode error %.2e" % (name, len(db.blocks), worst))
    del src, dst, ps, pd, out, out_src, ws
    torch.cuda.empty_cache()


def test_llama2_7b_full_size(oracle):
    run_config(oracle, "llama2_7b", 6, 6, 8)


def test_llama3_8b_gqa_full_size(oracle):
    run_config(oracle, "llama3_8b_gqa", 10, 8, 32)


def test_llama2_13b_long_full_size(oracle):
    run_config(oracle, "llama2_13b_long", 4, 3, 1)
