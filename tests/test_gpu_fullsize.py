"""GPU parity at the benchmark's full sizes, in the launch configuration bench.py
times (library defaults), for the 7B-, 8B-GQA- and 13B-shaped configs.

Whole pools (128 GiB and more) cannot be brought to the host, so the checks are:
  * EVERY completely written destination block, in every plane, holds the
    generator's content of its source block (the definition of the move at block
    granularity, evaluated on the device); the same for the source blocks, which
    must still hold their own content;
  * EVERY partly written last block goes to the host and is compared bit for bit
    with the CPU oracle run on the regenerated source and destination blocks;
  * for the 7B and 8B-GQA configs ALL written blocks additionally go to the host
    and are compared with the CPU oracle run on regenerated inputs, request by
    request (the 13B config moves 100 GiB: there the oracle sees samples);
  * position-sensitive hashes of every (plane, block): the source pool is
    unchanged and exactly the allocated destination blocks changed;
  * the staging buffer against the oracle's pack on sampled (request, layer,
    token window) pieces, then unpack into a re-filled destination, all blocks
    checked again;
  * sampled decode outputs (request, layer, query head) within 2e-3 of the fp64
    oracle over the regenerated K/V rows, and decode over the destination bit-equal
    to decode over the source for every row.
"""
import concurrent.futures as cf

import numpy as np
import pytest
import torch

import kvm_workload as wl
import paper_2501_06709_amd as kvm
from kvm_workload import device as wl_device

from gpu_util import DEV, assert_blocks_equal_generator, full_and_partial, planes_view

pytestmark = pytest.mark.gpu
TOL = 2e-3


def setup(name, need_dst=True):
    w = wl.make(name)
    m = w.model
    torch.cuda.empty_cache()            # memory an earlier test's tensors left in torch's cache
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


def request_blocks(sb, db, r, k, B):
    nb = -(-int(k) // B)
    return (sb.blocks[sb.offsets[r]:sb.offsets[r] + nb].astype(np.int64),
            db.blocks[db.offsets[r]:db.offsets[r] + nb].astype(np.int64))


def all_written_blocks_on_device(w, m, src, dst, sb, db, k):
    """Every completely written destination block == generator(source block), and the
    source blocks themselves still == generator(source block): all planes, all blocks."""
    s_pos, _ = full_and_partial(sb.offsets, sb.blocks, k, m.B)
    d_pos, partial = full_and_partial(db.offsets, db.blocks, k, m.B)
    s_ids, d_ids = sb.blocks[s_pos], db.blocks[d_pos]
    assert len(s_ids) == len(d_ids)
    assert_blocks_equal_generator(dst, m, w.n_blocks_dst, d_ids, s_ids, w.seed, wl.STREAM_SRC,
                                  "destination")
    assert_blocks_equal_generator(src, m, w.n_blocks_src, s_ids, s_ids, w.seed, wl.STREAM_SRC, "source")
    return len(d_ids), partial


def partial_blocks_vs_oracle(oracle, w, m, src, dst, sb, db, partial):
    """Every partly written last block: all planes to the host, against the oracle."""
    sp, dp = planes_view(src, m, w.n_blocks_src), planes_view(dst, m, w.n_blocks_dst)
    st1 = oracle.canonical_strides(m.L, m.H, m.D, m.B, 1)
    for r, j, ns in partial:
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
        assert np.array_equal(got, exp), "request %d last block %d (-> %d, %d slots) differs" % (r, j, dblk, ns)


def request_vs_oracle(oracle, w, m, dst_planes_host, s_ids, d_ids, k, r):
    """One request's written blocks (host copy [2L][nb][run]) against the oracle run on
    regenerated inputs: a compact pool holding just this request."""
    nb = len(s_ids)
    mini_src = np.stack([wl.gen_blocks(w.seed, wl.STREAM_SRC, m, p, s_ids) for p in range(2 * m.L)])
    exp = np.zeros_like(mini_src)          # full blocks are overwritten entirely
    if int(k) % m.B:                       # the last block keeps its own bytes past slot k % B
        for p in range(2 * m.L):
            exp[p, nb - 1] = wl.gen_block(w.seed, wl.STREAM_DST, m, p, int(d_ids[-1]))
    st = oracle.canonical_strides(m.L, m.H, m.D, m.B, nb)
    exp = exp.reshape(-1)
    oracle.migrate(mini_src.reshape(-1), st, exp, st, m.L, m.H, m.D, m.B, [0, nb], np.arange(nb), [0, nb],
                   np.arange(nb), [int(k)])
    assert np.array_equal(dst_planes_host.reshape(-1), exp), "request %d differs from the oracle" % r


def all_written_blocks_vs_oracle(oracle, w, m, dst, sb, db, k):
    """Brings every written destination block to the host and compares it with the
    oracle, request by request on worker threads (numpy and the C oracle release the
    interpreter lock)."""
    dp = planes_view(dst, m, w.n_blocks_dst)
    jobs = []
    for r in range(sb.n_req):
        if int(k[r]) == 0:
            continue
        s_ids, d_ids = request_blocks(sb, db, r, k[r], m.B)
        host = dp[:, torch.from_numpy(d_ids).to(DEV)].cpu().numpy().view(np.uint16)
        jobs.append((host, s_ids, d_ids, int(k[r]), r))
    with cf.ThreadPoolExecutor(16) as ex:
        list(ex.map(lambda j: request_vs_oracle(oracle, w, m, *j), jobs))
    return sum(len(j[1]) for j in jobs)


def sampled_blocks_vs_oracle(oracle, w, m, src, dst, sb, db, k, rng, n_samples):
    """Random written blocks plus the ones with the highest source and destination ids
    (largest byte offsets) through the oracle on regenerated blocks."""
    sp, dp = planes_view(src, m, w.n_blocks_src), planes_view(dst, m, w.n_blocks_dst)
    st1 = oracle.canonical_strides(m.L, m.H, m.D, m.B, 1)
    reqs = [r for r in range(sb.n_req) if k[r] > 0]
    picks = [(int(r), int(rng.integers(-(-int(k[r]) // m.B)))) for r in rng.choice(reqs, n_samples)]
    pos = [(r, j) for r in reqs for j in range(-(-int(k[r]) // m.B))]
    picks.append(max(pos, key=lambda rj: sb.blocks[sb.offsets[rj[0]] + rj[1]]))
    picks.append(max(pos, key=lambda rj: db.blocks[db.offsets[rj[0]] + rj[1]]))
    for r, j in picks:
        ns = min(m.B, int(k[r]) - j * m.B)
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


def staging_windows_vs_oracle(oracle, w, m, stage, sb, k, rng, n_samples, width=48):
    """Sampled (request, layer, token window) pieces of the staging buffer against the
    oracle's pack of that window on regenerated source blocks.  The windows include
    each request's first and last tokens."""
    st16 = stage.view(torch.int16)
    reqs = [r for r in range(sb.n_req) if k[r] > 0]
    base = np.concatenate([[0], np.cumsum(k.astype(np.int64))]) * (m.L * 2 * m.H * m.D)
    picks = []
    for r in reqs:
        picks += [(r, 0), (r, max(0, int(k[r]) - width))]
    picks += [(int(r), int(rng.integers(0, max(1, int(k[r]) - width)))) for r in rng.choice(reqs, n_samples)]
    for r, t0 in picks:
        t1 = min(int(k[r]), t0 + width)
        l = int(rng.integers(m.L))
        j0, j1 = t0 // m.B, -(-t1 // m.B)
        ids = sb.blocks[sb.offsets[r] + j0:sb.offsets[r] + j1].astype(np.int64)
        nb = len(ids)
        # compact one-layer source pool [1][kv][nb][H][B][D] holding the window's blocks
        mini = np.stack([wl.gen_blocks(w.seed, wl.STREAM_SRC, m, 2 * l + c, ids) for c in range(2)])
        st = oracle.canonical_strides(1, m.H, m.D, m.B, nb)
        exp = oracle.pack(mini.reshape(-1), st, 1, m.H, m.D, m.B, [0, nb], np.arange(nb),
                          [t1 - j0 * m.B], start=[t0 - j0 * m.B]).reshape(2, m.H, t1 - t0, m.D)
        n = int(k[r])
        for c in range(2):
            for h in range(m.H):
                at = int(base[r]) + (((l * 2 + c) * m.H + h) * n + t0) * m.D
                got = st16[at:at + (t1 - t0) * m.D].cpu().numpy().view(np.uint16).reshape(t1 - t0, m.D)
                assert np.array_equal(got, exp[c, h]), "staging (r=%d, l=%d, kv=%d, h=%d, t0=%d)" % (r, l, c, h, t0)


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


def hashes_show_only_the_table_changed(src, dst, w, m, src_hash, dst_hash, db):
    assert torch.equal(wl_device.plane_block_hashes(src, m, w.n_blocks_src), src_hash), "source pool changed"
    after = wl_device.plane_block_hashes(dst, m, w.n_blocks_dst)
    changed = (after != dst_hash).any(dim=0).cpu().numpy()
    written = np.zeros(w.n_blocks_dst, bool)
    written[db.blocks] = True
    assert not (changed & ~written).any(), "a block outside the destination table changed"
    assert changed[written].all(), "an allocated destination block did not change"


def run_config(oracle, name, n_block_samples, n_decode_samples, stage_requests, host_complete):
    w, m, src, dst, ps, pd, sb, db, lay = setup(name)
    rng = np.random.default_rng(7)
    src_hash = wl_device.plane_block_hashes(src, m, w.n_blocks_src)
    dst_hash = wl_device.plane_block_hashes(dst, m, w.n_blocks_dst)

    kvm.kvm_migrate(ps, sb, pd, db)
    torch.cuda.synchronize()
    hashes_show_only_the_table_changed(src, dst, w, m, src_hash, dst_hash, db)
    n_full, partial = all_written_blocks_on_device(w, m, src, dst, sb, db, w.k)
    partial_blocks_vs_oracle(oracle, w, m, src, dst, sb, db, partial)
    assert n_full + len(partial) == len(db.blocks)
    if host_complete:
        assert all_written_blocks_vs_oracle(oracle, w, m, dst, sb, db, w.k) == len(db.blocks)
    sampled_blocks_vs_oracle(oracle, w, m, src, dst, sb, db, w.k, rng, n_block_samples)

    # staged path into a re-filled destination: the staging buffer sampled against the
    # oracle's pack, then every block of the end state again
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
    staging_windows_vs_oracle(oracle, w, m, stage, sb2, k2, rng, 6)
    del stage
    n_full2, partial2 = all_written_blocks_on_device(w, m, src, dst, sb2, db2, k2)
    partial_blocks_vs_oracle(oracle, w, m, src, dst, sb2, db2, partial2)
    assert torch.equal(wl_device.plane_block_hashes(src, m, w.n_blocks_src), src_hash)
    # blocks of requests that were not staged hold the destination's own fill again
    rest = np.concatenate([db.blocks[db.offsets[r]:db.offsets[r + 1]] for r in range(sb.n_req)
                           if k2[r] == 0] + [np.zeros(0, np.int32)])
    assert_blocks_equal_generator(dst, m, w.n_blocks_dst, rest, rest, w.seed, wl.STREAM_DST, "unstaged")

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
    print("%s: %d blocks moved (%d partly), worst sampled decode error %.2e"
          % (name, len(db.blocks), len(partial), worst))
    del src, dst, ps, pd, out, out_src, ws
    torch.cuda.empty_cache()


def test_llama2_7b_full_size(oracle):
    run_config(oracle, "llama2_7b", 6, 6, 8, host_complete=True)


def test_llama3_8b_gqa_full_size(oracle):
    run_config(oracle, "llama3_8b_gqa", 10, 8, 32, host_complete=True)


def test_llama2_13b_long_full_size(oracle):
    run_config(oracle, "llama2_13b_long", 24, 3, 1, host_complete=False)


def test_llama2_13b_long_all_four_requests_through_one_staging_buffer(oracle):
    """All four 32768-token requests packed by ONE kvm_pack call into a 100 GiB
    staging buffer (26 million 4 KiB workgroups in one launch: more than one grid
    dimension holds), sampled against the oracle, then unpacked by one kvm_unpack call
    into a fresh destination pool where every block is checked.  The pools take turns
    in HBM: source + staging, then staging + destination."""
    w = wl.make("llama2_13b_long")
    m = w.model
    n_stage = int(w.k.astype(np.int64).sum()) * m.bytes_per_token
    torch.cuda.empty_cache()
    free_b, _ = torch.cuda.mem_get_info()
    if n_stage + w.n_blocks_dst * m.block_bytes + (12 << 30) > free_b:
        pytest.skip("needs %.0f GiB of HBM" % ((n_stage + w.n_blocks_dst * m.block_bytes) / 2**30))
    rng = np.random.default_rng(11)
    lay_s = kvm.kvm_layout_canonical(m.L, m.H, m.Hq, m.D, m.B, m.dtype, w.n_blocks_src)
    lay_d = kvm.kvm_layout_canonical(m.L, m.H, m.Hq, m.D, m.B, m.dtype, w.n_blocks_dst)
    s_off, s_blk = w.src_csr()
    sb = kvm.Batch(s_off, s_blk, w.k, torch.from_numpy(s_blk).to(DEV))
    src = torch.empty(kvm.kvm_pool_span_bytes(lay_s, w.n_blocks_src), dtype=torch.uint8, device=DEV)
    wl_device.fill_pool(src, m, w.n_blocks_src, w.seed, wl.STREAM_SRC)
    stage = torch.empty(n_stage + 4096, dtype=torch.uint8, device=DEV)
    stage[n_stage:].fill_(0xA5)                                     # guard behind the buffer
    kvm.kvm_pack(kvm.Pool(src, w.n_blocks_src, lay_s), sb, stage, staging_bytes=n_stage)
    torch.cuda.synchronize()
    assert bool((stage[n_stage:] == 0xA5).all()), "kvm_pack wrote past the staging buffer"
    staging_windows_vs_oracle(oracle, w, m, stage, sb, w.k, rng, 24)
    del src
    torch.cuda.empty_cache()

    dst = torch.empty(kvm.kvm_pool_span_bytes(lay_d, w.n_blocks_dst), dtype=torch.uint8, device=DEV)
    fl = kvm.FreeList(w.n_blocks_dst, w.dst_occupied)
    nbk = w.n_dst_blocks()
    ids = fl.alloc(sum(nbk))
    d_off = np.zeros(len(nbk) + 1, np.int32)
    d_off[1:] = np.cumsum(nbk)
    db = kvm.Batch(d_off, ids, w.k, torch.from_numpy(ids).to(DEV))
    pd = kvm.Pool(dst, w.n_blocks_dst, lay_d)
    untouched = np.flatnonzero(w.dst_occupied).astype(np.int32)
    for linear in (0, 2):                 # unpack cut by pool block (shipped) and along the staging buffer
        wl_device.fill_pool(dst, m, w.n_blocks_dst, w.seed, wl.STREAM_DST)
        try:
            kvm.kvm_set_option("copy.stage_linear", linear if linear else -1)
            kvm.kvm_unpack(stage, pd, db, staging_bytes=n_stage)
        finally:
            kvm.kvm_set_option("reset", 0)
        torch.cuda.synchronize()
        assert_blocks_equal_generator(dst, m, w.n_blocks_dst, ids, s_blk[:len(ids)], w.seed, wl.STREAM_SRC,
                                      "destination after unpack (stage_linear %d)" % linear)
        assert_blocks_equal_generator(dst, m, w.n_blocks_dst, untouched, untouched, w.seed, wl.STREAM_DST,
                                      "occupied destination blocks")
    del stage, dst
    torch.cuda.empty_cache()
